// C-ABI entry points of the ABFT GEMM library (see include/abft.h) and the small
// kernels around the GEMM: weight checksum (offline, paper Sec. 2.5), activation
// checksum fused with the checksum dot product (Sec. 2.4 steps 1-2) and the final
// reduction + comparison (Sec. 2.4 steps 3-4, Sec. 2.5 step 5).
#include <hip/hip_runtime.h>

#include <cmath>
#include <type_traits>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <cstring>
#include <atomic>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/abft.h"
#include "gemm_configs.h"
#include "mlp_chain.h"

using namespace abft;

namespace {

// ------------------------------------------------------------------------- //
// constants of the method as built here
// ------------------------------------------------------------------------- //
// Tolerance: tau = C_TOL * (2^-24 * sqrt(K) + u_chi) * ||C_S||_F + C_BIAS * 2^-24 * K * ||C_S||_1
// (the last term for the global scheme only).  2^-24 is the unit
// roundoff of the fp32 accumulators; an accumulator that takes K products carries a
// random-walk error ~ 2^-24 sqrt(K) |C_ij| / 2.4 and the errors of the entries add in
// quadrature under the output summation.  u_chi covers the tile checksum operand of the
// thread-level scheme, which is exact to 22 (fp16: two pieces) / 24 (bf16: three
// pieces) bits of the fp32 column sums.  The ||.||_1 term covers a small coherent bias of the
// matrix unit's accumulation (measured: up to 2e-4 * 2^-24 * K per entry, same sign for all
// entries of a tile with same-sign operands); in the thread-level scheme both sides of the
// comparison come out of the same unit and the bias cancels.
constexpr double C_TOL = 8.0;
constexpr double C_BIAS = 1.0e-3;
constexpr double U_ACC = 5.9604644775390625e-08;  // 2^-24
constexpr double U_CHI_F16 = 2.384185791015625e-07;  // 2^-22
constexpr double U_CHI_BF16 = 1.1920928955078125e-07;  // 2^-23
// ABFT_THREAD_HALF / ABFT_TWOSIDED add checksums in the operand type: every such add rounds to
// u_half = 2^-11 (fp16) / 2^-8 (bf16).  The errors of the B-side sums enter the comparison
// weighted with the column sums of the A tile, which are at most sqrt(tile rows) times the
// columns' norms (and the other way round for the A-side sums of the two-sided scheme):
//   tau += C_HALF * u_half * sqrt(n_B * tile_m + n_A * tile_n) * ||C_S||_F
// with n_B / n_A the number of adds per checksum element (fragments per wavefront tile - 1).
constexpr double C_HALF = 4.0;
constexpr double U_HALF_F16 = 4.8828125e-04, U_HALF_BF16 = 3.90625e-03;


// MI355X spec-sheet peaks (dense) and HBM3E bandwidth
constexpr double PEAK_F16 = 2516.6e12, PEAK_I8 = 5033.2e12, HBM_BW = 8.0e12;
double g_cmr_override[3] = {0.0, 0.0, 0.0};

// optional events recorded around the GEMM kernel launch (abft_set_kernel_events)
thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;

// Scratch of abft_gemm_static: one array per GPU the library runs on, held until the process
// ends.  The name below is only a host-side stand-in for the array; its device address is asked
// for once per device (scratch_of_current_device) and that pointer is what kernels are given.
constexpr size_t STATIC_SCRATCH_BYTES = 8u << 20;
__device__ __align__(256) unsigned char g_static_scratch[STATIC_SCRATCH_BYTES];
// product launches so far that took their activation checksums from the layer before (diagnostics)
std::atomic<long long> g_handover_launches{0};
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};
std::mutex g_scratch_mutex;

// device address of this GPU's copy of the scratch array (null: the runtime refused)
void* scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

inline int esize(int dt) { return dt == ABFT_I8 ? 1 : 2; }
inline int csize(int dt) { return dt == ABFT_I8 ? 4 : 2; }
inline bool valid_dtype(int dt) { return dt == ABFT_F16 || dt == ABFT_BF16 || dt == ABFT_I8; }
inline long long cdiv(long long a, long long b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ------------------------------------------------------------------------- //
// tile configuration choice (host logic)
// ------------------------------------------------------------------------- //
// mode: the scheme the product will run with (thread-level prefers wavefront tiles that are
// wide in N: one checksum MFMA per TN real ones); force >= 0 pins a configuration (tuning aid,
// environment variable ABFT_FORCE_CFG).
int pick_cfg(int M, int N, int K, int dt, bool aligned16, int mode) {
    // (every wavefront-level scheme is checked per wavefront tile: the same tiles)
    if (mode == ABFT_REPLICA || mode == ABFT_THREAD_HALF || mode == ABFT_TWOSIDED) mode = ABFT_THREAD;
    if (mode == ABFT_GLOBAL_WEIGHTED) mode = ABFT_GLOBAL;
    static const int force = [] {
        const char* e = std::getenv("ABFT_FORCE_CFG");
        return e ? std::atoi(e) : -1;
    }();
    // the direct-to-LDS kernel needs whole k tiles of 128 bytes; the streaming kernel takes any whole
    // number of 16-byte chunks (a variant of it fills a short last tile up with zeros)
    const bool fast_ok = aligned16 && ((long long)K * esize(dt)) % 128 == 0;
    const bool force_fits = force >= 0 && force < CFG_COUNT &&
                            (fast_ok || !cfg_info_host(force).fast || (aligned16 && cfg_is_stream(force)));
    // (the 256 x 256 tile carries no wavefront-level scheme: a forced choice of it does not apply to those)
    if (force_fits && !((force == CFG_F256W || force == CFG_F256N || force == CFG_F256S || force == CFG_F128E) && mode == ABFT_THREAD)) return force;
    if (M <= 16 && !aligned16) return CFG_G16;
    auto tiles = [&](int id) {
        CfgInfo ci = cfg_info_host(id);
        return cdiv(M, ci.bm) * cdiv(N, ci.bn);
    };
    if (aligned16) {
        // fill the 256 compute units before growing the tile
        // (thread-level: the 128 x 128 tile of wide wavefront tiles; the 256 x 256 one would spill)
        // (a single k tile: the 128 x 128 tile, of which several fit a compute unit at once)
        const long long nkt_all = cdiv((long long)K * esize(dt), 128);
        // The 256 x 256 tile runs one workgroup per compute unit, in rounds of 256: it is taken when
        // the rounds are at least 70 % full (288 tiles would leave the second round of 6000 x 3072 x
        // 768 almost empty: 58 us against 48 us on 128 x 128 tiles), from 192 tiles on when the k loop
        // is eight tiles long or more (50176 x 256 x 512, 12544 x 1024 x 512: 196 tiles each), else from 224.
        const long long t256 = tiles(CFG_F256W);
        const bool rounds_full = t256 * 10 >= cdiv(t256, 256) * 256 * 7;
        if (fast_ok && N > 128 && nkt_all > 1 && rounds_full && (t256 >= 224 || (t256 >= 192 && nkt_all >= 8)))
            return mode == ABFT_THREAD ? CFG_F128T : CFG_F256W;
        // About one 256 x 128 tile per compute unit (one round, more than half full) with a k loop
        // of six tiles or more: that tile keeps three stages in LDS and asks the vector memory
        // path for three quarters of what 128 x 128 tiles ask per MFMA (2048 x 4096 x 4096: 70 us
        // against 77 us; 1536 x 4096 x 4096: 59 against 65; 2048 x 3072 x 4096: 56 against 63;
        // 144 tiles, 1152 x 4096 x 4096: 52 against 57; 128 tiles, 1024 x 4096 x 4096: 53 against 48;
        // k loop of four tiles: level).  Its wavefront tiles carry no wavefront-level scheme.
        const long long t256n = tiles(CFG_F256N);
        if (fast_ok && mode != ABFT_THREAD && N >= 128 && nkt_all >= 6 && t256n >= 144 && t256n <= 256) return CFG_F256N;
        // Outputs of at most 64 columns and very many rows (ResNet-50's first stage at batch 64: 200704
        // rows): 256 x 64 tiles with three stages.  3 x 3 convolution 64 -> 64: 46 us against 52 us
        // unprotected, 52 against 63 global; K = 64: 17 against 23 us global, level unprotected; k loops
        // of two to five tiles: slower unprotected (33 against 30 us at K = 256).
        if (fast_ok && mode != ABFT_THREAD && N <= 64 && N > 32 && M >= 65536 &&
            (nkt_all >= 6 || (nkt_all == 1 && mode == ABFT_GLOBAL)))
            return CFG_F256S;
        const bool fills128 = tiles(CFG_F128) >= 128;
        if (fast_ok && fills128 && N < 128) return CFG_F128T;  // narrow outputs: every wavefront spans all columns
        // Few tiles: the time is the latency of a workgroup's k loop and the rate at which one
        // compute unit can stream its operands, so the streaming configurations take over (no
        // barriers in the k loop, four wavefronts sharing the k tiles): the smallest tile that
        // still fits the chip in one round of workgroups, 64 x 64 for up to two rounds (that one
        // only with a k loop of at least one tile per wavefront, sixteen tiles (thread-level: eight) for a second round:
        // the idle wavefronts of a short loop cost more than the barriers they save; 3000 x 384 x
        // 384 takes 9.9 us on 282 such tiles, 8.2 us on 64 x 128 tiles).  (On the 32 x 32 tile the thread-level
        // scheme's checksum operand is the B fragment itself: no vector work at all.)
        if (tiles(CFG_S32) <= 256) return CFG_S32;
        if (tiles(CFG_S64) <= 256) return CFG_S64;
        if (tiles(CFG_S128) <= 256 ? nkt_all >= 4 : (tiles(CFG_S128) <= 512 && nkt_all >= (mode == ABFT_THREAD ? 8 : 16))) return CFG_S128;
        if (fast_ok) {
            // (thread-level: the wide wavefront tiles pay off once two workgroups share a compute unit;
            // with at most one per unit the 64 x 64 wavefront tiles' cheaper checksum wins: 1536 x 2048 x
            // 2048 takes 37 us against 42 us, 640 x 5120 x 1280 26 us against 30 us)
            // At most one 128 x 128 tile per compute unit (one round): eight wavefronts of 32 x 64 on the
            // 16x16x32 shapes with three stages instead of four wavefronts of 64 x 64 with two: the second
            // wavefront per SIMD and the deeper pipeline hide what a second workgroup would (1024 x 4096 x
            // 4096: 40-43 us against 46-48; 2048^3: 22 against 26; 12544 x 256 x 2304: 25 against 28;
            // global the same tenth).  Two rounds: slower (3072 x 4096 x 4096: 115 against 91 us on two
            // workgroups per unit).  No wavefront-level scheme on it.
            if (fills128 && mode != ABFT_THREAD && tiles(CFG_F128) <= 256 && nkt_all >= 4) return CFG_F128E;
            if (fills128) return (nkt_all <= 1 || (mode == ABFT_THREAD && tiles(CFG_F128) > 256)) ? CFG_F128T : CFG_F128;
            return CFG_F64T;
        }
    }
    if (tiles(CFG_G128) >= 192) return CFG_G128;
    if (tiles(CFG_G64) >= 1024) return CFG_G128;
    return CFG_G64;
}

// ------------------------------------------------------------------------- //
// auxiliary kernels
// ------------------------------------------------------------------------- //
struct PreArgs {
    const char* A;
    int M, K;
    long long lda;
    int vec;
    int conv, H, W, Cin, KH, KW, stride, pad, OH, OW;
    long long imgpitch, rowpitch;  // as in GemmArgs
    int pix;
    void* alpha_out;      // K doubles / int64: the plain checksum (single-slab launches only), or null
    int rows_per_slab;    // rows of one row block of the product's tiling
    int rows_per_block;   // rows one workgroup sums; divides rows_per_slab
    const void* beta;     // K x nb (k-major) weight checksums per column block, or null
    void* partial_dots;   // [slab][nb][subs * gridDim.x] partial checksum dot products, or null
    int nb;
};

// Activation checksum alpha_s[k] = sum over the rows m of slab s of A[m][k] (Sec. 2.4
// step 1), one slab per row block of the product's workgroup tiling.
// Block = 32 chunk columns x 8 row lanes.
template <int DT>
__global__ __launch_bounds__(256) void act_checksum_kernel(const PreArgs p) {
    constexpr int ESIZE = DT == DT_I8 ? 1 : 2;
    constexpr int EPC = 16 / ESIZE;
    typedef typename std::conditional<DT == DT_I8, long long, double>::type Wide;
    __shared__ Wide red[8][32][EPC];

    const int tid = threadIdx.x, tx = tid & 31, ty = tid >> 5;
    const int k0 = (blockIdx.x * 32 + tx) * EPC;
    const int subs = p.rows_per_slab / p.rows_per_block;
    const int slab = blockIdx.y / subs, sub = blockIdx.y - slab * subs;
    const int row_begin = slab * p.rows_per_slab + sub * p.rows_per_block;
    const int row_end = min(p.M, row_begin + p.rows_per_block);

    // per-element filter tap for the implicit-GEMM view (k is fixed per thread)
    int e_off[EPC], e_kh[EPC], e_kw[EPC];
    if (p.conv) {
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
            int k = k0 + e;
            int tap = k / p.Cin;
            e_off[e] = k - tap * p.Cin;
            e_kh[e] = tap / p.KW;
            e_kw[e] = tap - e_kh[e] * p.KW;
        }
    }

    Wide s[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) s[e] = 0;

    __shared__ Wide alpha_s[32 * EPC];
    // Rows whose chunks cannot be read whole (K or the leading dimension is no multiple of a
    // chunk): one element per thread and row instead.  Thread t takes column t % kb of the kb
    // columns of a pass and every nrg-th row, so that adjacent lanes read adjacent elements of a
    // row and the loads of one thread do not wait for each other.
    const bool by_element = !p.conv && !p.vec;
    if (by_element) {
        const int kbase = blockIdx.x * 32 * EPC;
        const int kb_all = min(32 * EPC, p.K - kbase);   // columns of this block
        Wide* part = &red[0][0][0];
        Wide* out = reinterpret_cast<Wide*>(p.alpha_out);
        for (int c0 = 0; c0 < 32 * EPC; c0 += 256) {     // (int8 blocks span 512 columns: two passes)
            const int kb = min(256, kb_all - c0);        // columns of this pass; none left: <= 0
            Wide acc = 0;
            if (kb > 0) {
                const int nrg = 256 / kb, col = tid % kb, rg = tid / kb;
                if (rg < nrg) {
                    const char* src = p.A + (long long)(kbase + c0 + col) * ESIZE;
                    for (int m0 = row_begin + rg; m0 < row_end; m0 += 8 * nrg) {
                        Wide v[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const int m = m0 + u * nrg;
                            const int mc = m < row_end ? m : m0;   // a valid row; its value is dropped below
                            const char* q = src + (long long)mc * p.lda * ESIZE;
                            Wide x;
                            if constexpr (DT == DT_F16) x = (double)(float)*reinterpret_cast<const _Float16*>(q);
                            else if constexpr (DT == DT_BF16) x = (double)(float)*reinterpret_cast<const __bf16*>(q);
                            else x = (long long)*reinterpret_cast<const signed char*>(q);
                            v[u] = m < row_end ? x : (Wide)0;
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) acc += v[u];
                    }
                }
            }
            part[tid] = acc;
            __syncthreads();
            Wide a = 0;
            if (tid < kb) {
                const int nrg = 256 / kb;
                for (int g = 0; g < nrg; ++g) a += part[g * kb + tid];
                if (out) out[kbase + c0 + tid] = a;
            }
            alpha_s[c0 + tid] = a;
            __syncthreads();
        }
    }
    for (int m0 = row_begin + ty; m0 < row_end && !by_element; m0 += 64) {
        // int8: up to eight rows are summed in int32 first (exact); fp16 / bf16 values are
        // widened and added in fp64 one by one, so the checksum side carries no rounding
        // that could show up in the comparison
        typename std::conditional<DT == DT_I8, int, double>::type f[EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) f[e] = 0;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int m = m0 + 8 * u;
            if (m >= row_end || k0 >= p.K) continue;
            i32x4 v = {0, 0, 0, 0};
            if (!p.conv) {
                const char* src = p.A + ((long long)m * p.lda + k0) * ESIZE;
                v = p.vec ? ld16(src) : gather16<ESIZE>(src, ESIZE, p.K - k0);
            } else {
                int img = m / (p.OH * p.OW);
                int rem = m - img * (p.OH * p.OW);
                int oh = rem / p.OW, ow = rem - oh * p.OW;
                int ih0 = oh * p.stride - p.pad, iw0 = ow * p.stride - p.pad;
                const char* base = p.A + (long long)img * p.imgpitch * ESIZE;
                if (p.vec) {
                    int ih = ih0 + e_kh[0], iw = iw0 + e_kw[0];
                    if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W)
                        v = ld16(base + ((long long)ih * p.rowpitch + (long long)iw * p.pix + e_off[0]) * ESIZE);
                } else {
#pragma unroll
                    for (int e = 0; e < EPC; ++e) {
                        int ih = ih0 + e_kh[e], iw = iw0 + e_kw[e];
                        unsigned x = 0;
                        if (k0 + e < p.K && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W) {
                            const char* src = base + ((long long)ih * p.rowpitch + (long long)iw * p.pix + e_off[e]) * ESIZE;
                            x = ESIZE == 2 ? (unsigned)*reinterpret_cast<const unsigned short*>(src)
                                           : (unsigned)*reinterpret_cast<const unsigned char*>(src);
                        }
                        if (ESIZE == 2) v[e >> 1] |= (int)(x << (16 * (e & 1)));
                        else v[e >> 2] |= (int)(x << (8 * (e & 3)));
                    }
                }
            }
            if constexpr (DT == DT_F16) {
                f16x8 h = bitcast<f16x8>(v);
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] += (double)(float)h[e];
            } else if constexpr (DT == DT_BF16) {
                bf16x8 h = bitcast<bf16x8>(v);
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] += (double)(float)h[e];
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) f[e] += (int)(signed char)(v[e >> 2] >> (8 * (e & 3)));
            }
        }
#pragma unroll
        for (int e = 0; e < EPC; ++e) s[e] += (Wide)f[e];
    }
    if (!by_element) {
#pragma unroll
        for (int e = 0; e < EPC; ++e) red[ty][tx][e] = s[e];
    }
    __syncthreads();
    if (ty == 0 && !by_element) {
        Wide* out = reinterpret_cast<Wide*>(p.alpha_out);
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
            Wide a = 0;
            for (int y = 0; y < 8; ++y) a += red[y][tx][e];
            alpha_s[tx * EPC + e] = (k0 + e < p.K) ? a : (Wide)0;
            if (out && k0 + e < p.K) out[k0 + e] = a;
        }
    }
    if (!p.partial_dots) return;
    // Sec. 2.4 step 2, fused: this block's share of the checksum dot products
    //   P[slab][j][sub, chunk] = sum over the block's rows and k range of A[m][k] * beta_j[k]
    // lanes run over the column blocks j (beta is k-major, so these reads are contiguous),
    // the 8 lane groups split the k range
    __syncthreads();
    const int kbase = blockIdx.x * 32 * EPC;
    const int kcount = min(32 * EPC, p.K - kbase);
    const Wide* beta = reinterpret_cast<const Wide*>(p.beta);
    Wide* red2 = &red[0][0][0];  // reuse: 8 x 32 values
    const int n_parts = subs * gridDim.x;
    Wide* pout = reinterpret_cast<Wide*>(p.partial_dots) + (long long)slab * p.nb * n_parts + sub * gridDim.x + blockIdx.x;
    for (int jb = 0; jb < p.nb; jb += 32) {
        const int j = jb + tx;
        Wide acc = 0;
        if (j < p.nb) {
            // 32 * EPC / 8 values of k per thread, loaded in independent batches of eight
            const Wide* bj = beta + (long long)kbase * p.nb + j;
            for (int k0b = ty; k0b < 32 * EPC; k0b += 64) {
                Wide bv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int k = k0b + 8 * u;
                    bv[u] = k < kcount ? bj[(long long)k * p.nb] : (Wide)0;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) acc += alpha_s[k0b + 8 * u] * bv[u];
            }
        }
        __syncthreads();
        red2[ty * 32 + tx] = acc;
        __syncthreads();
        if (ty == 0 && j < p.nb) {
            Wide tot = 0;
            for (int y = 0; y < 8; ++y) tot += red2[y * 32 + tx];
            pout[(long long)j * n_parts] = tot;
        }
    }
}

// Weight checksum per block of columns: beta_b[k] = sum over the columns n of block b of
// B[k][n] (Sec. 2.5, offline), for any storage order (element strides).
// Block = 32 values of k x 8 lanes over n; blockIdx.y = column block.  Not tuned: offline.
template <int DT>
__global__ __launch_bounds__(256) void weight_checksum_kernel(const char* B, int K, int N, long long sn,
                                                              long long sk, int block_n, int wnorm, void* beta,
                                                              char* beta_k, char* beta_p, char* beta_r) {
    constexpr int ESIZE = DT == DT_I8 ? 1 : 2;
    typedef typename std::conditional<DT == DT_I8, long long, double>::type Wide;
    __shared__ Wide red[2][8][32];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int k = blockIdx.x * 32 + tx;
    const int n_begin = blockIdx.y * block_n, n_end = min(N, n_begin + block_n);
    // s: the plain checksum of the block's columns; sv: the same with column j of the block
    // weighted j + 1 (int8) or (j + 1) / wnorm (floating point; wnorm: the nominal block width, also
    // where N cuts the block short), the second of the independent linear combinations of Sec. 2.4's
    // last paragraph
    Wide s = 0, sv = 0;
    if (k < K) {
        for (int n = n_begin + ty; n < n_end; n += 8) {
            const char* src = B + ((long long)n * sn + (long long)k * sk) * ESIZE;
            Wide x;
            if constexpr (DT == DT_F16) x = (double)(float)*reinterpret_cast<const _Float16*>(src);
            else if constexpr (DT == DT_BF16) x = (double)(float)*reinterpret_cast<const __bf16*>(src);
            else x = (long long)*reinterpret_cast<const signed char*>(src);
            s += x;
            if constexpr (DT == DT_I8) sv += x * (n - n_begin + 1);
            else sv += x * ((double)(n - n_begin + 1) / (double)wnorm);
        }
    }
    red[0][ty][tx] = s;
    red[1][ty][tx] = sv;
    __syncthreads();
    if (ty == 0 && k < K) {
        Wide a = 0, av = 0;
        for (int y = 0; y < 8; ++y) {
            a += red[0][y][tx];
            av += red[1][y][tx];
        }
        reinterpret_cast<Wide*>(beta)[(long long)k * gridDim.y + blockIdx.y] = a;
        // second copy, per column block along k, for the in-kernel checksum dot product of the
        // direct-to-LDS kernel: floats, or (int8) balanced base-256 digits, K low then K high;
        // third copy (8 bytes per k and block) for the streaming kernel's matrix-unit form: fp16:
        // four planes of K halves, hi = fl16(beta), lo = fl16((beta - hi) 2^11), and the same two
        // pieces of the column-weighted checksum; int8: four planes of K digits of the
        // column-weighted checksum (balanced base 256, least significant first)
        // fourth copy, for the direct-to-LDS kernel: per block and k tile of that kernel (64 values of k;
        // int8: 128) a record of 1 KB -- fp16: 64 halves fl16(beta), 64 halves fl16((beta - hi) 2^11), then
        // (at byte 256) 64 floats; bf16: the 64 floats; int8: 128 low digits, 128 high digits
        constexpr int KT = DT == DT_I8 ? 128 : 64;
        char* rec = beta_r + ((long long)blockIdx.y * ((K + KT - 1) / KT) + k / KT) * 1024;
        const int kin = k % KT;
        if constexpr (DT == DT_I8) {
            const long long lo = (long long)(signed char)(a & 0xff);
            const long long hi = (a - lo) >> 8;
            signed char* d = reinterpret_cast<signed char*>(beta_k) + (long long)blockIdx.y * 2 * K;
            d[k] = (signed char)lo;
            d[K + k] = (signed char)(hi < -128 ? -128 : (hi > 127 ? 127 : hi));
            reinterpret_cast<signed char*>(rec)[kin] = d[k];
            reinterpret_cast<signed char*>(rec)[128 + kin] = d[K + k];
            signed char* dv = reinterpret_cast<signed char*>(beta_p) + (long long)blockIdx.y * 8 * K;
            long long rest = av;
            for (int q = 0; q < 4; ++q) {
                const long long digit = (long long)(signed char)(rest & 0xff);
                dv[(long long)q * K + k] = (signed char)digit;
                rest = (rest - digit) >> 8;
            }
        } else {
            reinterpret_cast<float*>(beta_k)[(long long)blockIdx.y * K + k] = (float)a;
            reinterpret_cast<float*>(rec + 256)[kin] = (float)a;
            if constexpr (DT == DT_F16) {
                _Float16* pl = reinterpret_cast<_Float16*>(beta_p) + (long long)blockIdx.y * 4 * K;
                const _Float16 hi = (_Float16)(float)a;
                pl[k] = hi;
                pl[K + k] = (_Float16)(((float)a - (float)hi) * 2048.f);
                reinterpret_cast<_Float16*>(rec)[kin] = pl[k];
                reinterpret_cast<_Float16*>(rec + 128)[kin] = pl[K + k];
                const _Float16 vhi = (_Float16)(float)av;
                pl[2 * K + k] = vhi;
                pl[3 * K + k] = (_Float16)(((float)av - (float)vhi) * 2048.f);
            }
        }
    }
}

// ------------------------------------------------------------------------- //
// Convolutions with few input channels (ResNet's first layer: Cin = 3), lowered to row
// segments.  For a filter row kh the KW taps x Cin channels are one contiguous run of the
// input row, so k is re-ordered as (kh, run position) with every run padded to whole 16-byte
// chunks, the input is copied once with its zero border (so no chunk needs masking) and the
// product reads whole chunks instead of gathering single elements.
// ------------------------------------------------------------------------- //
// padded copy of the NHWC input: out[img][r][x] (row pitch rowp elements), r over H + 2 pad rows,
// x over the padded row; one 16-byte chunk per thread
template <int ESIZE>
__global__ __launch_bounds__(256) void conv_pad_kernel(const char* x, char* out, int H, int WC, int pad, int padC,
                                                      int Hp, long long rowp, long long chunks_per_row,
                                                      long long total_chunks) {
    constexpr int EPC = 16 / ESIZE;
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total_chunks) return;
    const long long row = t / chunks_per_row;
    const long long e0 = (t - row * chunks_per_row) * EPC;
    const long long img = row / Hp;
    const int ih = (int)(row - img * Hp) - pad;
    i32x4 v = {0, 0, 0, 0};
    if (ih >= 0 && ih < H) {
        const char* src = x + ((img * H + ih) * (long long)WC) * ESIZE;
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
            const long long xe = e0 + e - padC;
            unsigned val = 0;
            if (xe >= 0 && xe < WC)
                val = ESIZE == 2 ? (unsigned)*reinterpret_cast<const unsigned short*>(src + xe * 2)
                                 : (unsigned)*reinterpret_cast<const unsigned char*>(src + xe);
            if (ESIZE == 2) v[e >> 1] |= (int)(val << (16 * (e & 1)));
            else v[e >> 2] |= (int)(val << (8 * (e & 3)));
        }
    }
    *reinterpret_cast<i32x4*>(out + (row * rowp + e0) * ESIZE) = v;
}

// weights in the lowered order: out[n][kh * segp + r] = B[k = (kh KW + r / Cin) Cin + r % Cin][n] for
// r < KW Cin and kh < KH, else 0
template <int ESIZE>
__global__ __launch_bounds__(256) void conv_weights_kernel(const char* B, long long sn, long long sk, char* out, int N,
                                                          int Kp, int segp, int seg, int KH) {
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= (long long)N * Kp) return;
    const int n = (int)(t / Kp), kp = (int)(t - (long long)n * Kp);
    const int kh = kp / segp, r = kp - kh * segp;
    if (ESIZE == 2) {
        unsigned short v = 0;
        if (r < seg && kh < KH) v = *reinterpret_cast<const unsigned short*>(B + ((long long)n * sn + (long long)(kh * seg + r) * sk) * 2);
        reinterpret_cast<unsigned short*>(out)[t] = v;
    } else {
        unsigned char v = 0;
        if (r < seg && kh < KH) v = *reinterpret_cast<const unsigned char*>(B + ((long long)n * sn + (long long)(kh * seg + r) * sk));
        reinterpret_cast<unsigned char*>(out)[t] = v;
    }
}

// ------------------------------------------------------------------------- //
// host helpers
// ------------------------------------------------------------------------- //
struct Problem {
    int M, N, K, dtype, b_layout;
    const void* A;
    long long lda;
    const void* B;
    long long ldb;
    void* C;
    long long ldc;
    bool conv;
    abft_conv_t cg;
    int OH, OW;
    long long imgpitch, rowpitch;  // conv: input element (img, ih, iw, c) at img*imgpitch + ih*rowpitch + iw*pix + c
    int pix;
    int tol_K;                     // K the tolerance is taken for (differs from K for a lowered convolution)
    int act;                       // abft_act_t applied to the stored values
    // chains of layers (Sec. 2.4 step 4): where this layer's epilogue leaves the activation checksums
    // of the NEXT layer (per 32-row block, leading dimension ld_alpha_out; see GemmArgs), whether it
    // did (not every kernel can), and the ones the layer before left for this layer's A
    float* alpha_out;
    long long ld_alpha_out;
    bool* alpha_emitted;
    const float* alpha_in;
};

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool a_vectorisable(const Problem& pr) {
    const int es = esize(pr.dtype);
    if (!aligned16(pr.A)) return false;
    // (a lowered convolution reads chunks at 4-byte aligned addresses: 16-byte loads still apply)
    if (pr.conv) return (pr.cg.Cin * es) % 16 == 0;
    return (pr.K * es) % 16 == 0 && (pr.lda * es) % 16 == 0;
}
bool b_vectorisable(const Problem& pr) {
    const int es = esize(pr.dtype);
    return pr.b_layout == ABFT_B_NK && aligned16(pr.B) && (pr.K * es) % 16 == 0 && (pr.ldb * es) % 16 == 0;
}

int conv_out(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

struct WsLayout {
    size_t off_pd, off_beta, total;
};

int pre_grid_x(int K, int dt) { return (int)cdiv(K, 32 * (16 / esize(dt))); }
// rows one workgroup of the activation-checksum kernel sums: a whole row block of the tiling
// when that still gives a few workgroups per compute unit, else 64 rows
int pre_rows_per_block(int bm, int M, int K) {
    if (bm <= 64) return bm;
    return cdiv(M, bm) * cdiv(K, 256) >= 512 ? bm : 64;
}

// Workspace of the global scheme for the tile configuration `cfg`: per-tile partial
// checksum dot products, per-column-block weight checksums
// (the last only used when the caller passes no precomputed ones).  Sized for any dtype.
// The weight-checksum buffer holds two copies: K x nb wide values (double / int64, k-major) for
// the activation-checksum kernel's dot products, then, 256-byte aligned, the per-block copy
// along k for the in-kernel dot product (4 bytes per k and block reserved).
size_t beta_k_offset(int K, int nb) { return align_up((size_t)K * nb * 8, 256); }
// third copy, 8 bytes per k and block: the columns of the extra operand with which the streaming
// kernel forms its dot products on the matrix unit (see weight_checksum_kernel)
size_t beta_p_offset(int K, int nb) { return beta_k_offset(K, nb) + align_up((size_t)K * nb * 4, 256); }
// fourth copy: one 1 KB record per block and k tile of the direct-to-LDS kernel (64 values of k; int8:
// 128), which one 16-byte-per-lane copy brings in with the operand tiles (see weight_checksum_kernel);
// sized for the shorter k tile
size_t beta_r_offset(int K, int nb) { return beta_p_offset(K, nb) + align_up((size_t)K * nb * 8, 256); }
size_t beta_total_bytes(int K, int nb) { return beta_r_offset(K, nb) + (size_t)nb * cdiv(K, 64) * 1024; }

WsLayout ws_layout(int M, int N, int K, int cfg) {
    CfgInfo ci = cfg_info_host(cfg);
    const size_t tm = (size_t)cdiv(M, ci.bm), tn = (size_t)cdiv(N, ci.bn);
    const size_t n_parts = (size_t)(ci.bm / (ci.bm < 64 ? ci.bm : 64)) * (size_t)cdiv(K, 256);  // upper bound
    WsLayout w;
    w.off_pd = 0;
    w.off_beta = align_up(w.off_pd + tm * tn * n_parts * 8, 256);
    w.total = align_up(w.off_beta + beta_total_bytes(K, (int)tn), 256);
    return w;
}

size_t ws_bytes_any_cfg(int M, int N, int K) {
    size_t best = 0;
    for (int id = 0; id < CFG_COUNT; ++id) {
        size_t t = ws_layout(M, N, K, id).total;
        if (t > best) best = t;
    }
    return best;
}

// extra coefficient of ||C_S||_F for the schemes that add checksums in the operand type, on
// wavefront tiles of tile_m x tile_n (MFMA blocks of mi rows / columns)
double tol_half_coeff(int dt, int mode, int tile_m, int tile_n, int mi) {
    if (dt == ABFT_I8 || (mode != ABFT_THREAD_HALF && mode != ABFT_TWOSIDED)) return 0.0;
    const double n_b = tile_n / mi - 1, n_a = mode == ABFT_TWOSIDED ? tile_m / mi - 1 : 0;
    return C_HALF * (dt == ABFT_F16 ? U_HALF_F16 : U_HALF_BF16) * std::sqrt(n_b * tile_m + n_a * tile_n);
}

double tol_coeff(int K, int dt, int mode) {
    if (dt == ABFT_I8) return 0.0;
    // (two fp32 accumulations compared, as in the thread-level scheme)
    if (mode == ABFT_REPLICA || mode == ABFT_THREAD_HALF || mode == ABFT_TWOSIDED) mode = ABFT_THREAD;
    double u_chi = 0.0;
    if (mode == ABFT_THREAD) u_chi = dt == ABFT_F16 ? U_CHI_F16 : U_CHI_BF16;
    return C_TOL * (U_ACC * std::sqrt((double)K) + u_chi);
}

// coefficient of the sum of magnitudes (global scheme only): covers the coherent bias of
// the matrix unit's accumulation, which grows like K per entry instead of sqrt(K)
double tol_bias_coeff(int K, int dt, int mode) {
    if (dt == ABFT_I8 || mode != ABFT_GLOBAL) return 0.0;
    return C_BIAS * U_ACC * (double)K;
}

double cmr_of(int dt) {
    if (g_cmr_override[dt] > 0.0) return g_cmr_override[dt];
    return (dt == ABFT_I8 ? PEAK_I8 : PEAK_F16) / HBM_BW;
}

double intensity(int M, int N, int K, int dt) {
    const double sa = esize(dt), sb = esize(dt), sc = csize(dt);
    const double m = M, n = N, k = K;
    return 2.0 * m * n * k / (sa * m * k + sb * k * n + sc * m * n);
}

int select_mode(int M, int N, int K, int dt) {
    return intensity(M, N, K, dt) > cmr_of(dt) ? ABFT_GLOBAL : ABFT_THREAD;
}

hipError_t launch_weight_checksum(int K, int N, const void* B, long long ldb, int layout, int dt, int block_n,
                                  void* beta_buf, hipStream_t st) {
    long long sn = layout == ABFT_B_NK ? ldb : 1, sk = layout == ABFT_B_NK ? 1 : ldb;
    const int wnorm = block_n > 0 ? block_n : N;
    if (block_n <= 0 || block_n > N) block_n = N;
    void* beta = beta_buf;
    char* beta_k = reinterpret_cast<char*>(beta_buf) + beta_k_offset(K, (int)cdiv(N, block_n));
    char* beta_p = reinterpret_cast<char*>(beta_buf) + beta_p_offset(K, (int)cdiv(N, block_n));
    char* beta_r = reinterpret_cast<char*>(beta_buf) + beta_r_offset(K, (int)cdiv(N, block_n));
    dim3 grid((unsigned)cdiv(K, 32), (unsigned)cdiv(N, block_n)), block(256);
    const char* b = reinterpret_cast<const char*>(B);
    if (dt == ABFT_F16)
        hipLaunchKernelGGL(weight_checksum_kernel<DT_F16>, grid, block, 0, st, b, K, N, sn, sk, block_n, wnorm, beta, beta_k, beta_p, beta_r);
    else if (dt == ABFT_BF16)
        hipLaunchKernelGGL(weight_checksum_kernel<DT_BF16>, grid, block, 0, st, b, K, N, sn, sk, block_n, wnorm, beta, beta_k, beta_p, beta_r);
    else
        hipLaunchKernelGGL(weight_checksum_kernel<DT_I8>, grid, block, 0, st, b, K, N, sn, sk, block_n, wnorm, beta, beta_k, beta_p, beta_r);
    return hipGetLastError();
}

hipError_t launch_act_checksum(const Problem& pr, void* alpha_out, int rows_per_slab, const void* beta, int nb,
                               void* partial_dots, hipStream_t st) {
    PreArgs a;
    std::memset(&a, 0, sizeof a);
    a.A = reinterpret_cast<const char*>(pr.A);
    a.M = pr.M;
    a.K = pr.K;
    a.lda = pr.lda;
    a.vec = a_vectorisable(pr) ? 1 : 0;
    a.conv = pr.conv ? 1 : 0;
    if (pr.conv) {
        a.imgpitch = pr.imgpitch; a.rowpitch = pr.rowpitch; a.pix = pr.pix;
        a.H = pr.cg.H; a.W = pr.cg.W; a.Cin = pr.cg.Cin; a.KH = pr.cg.KH; a.KW = pr.cg.KW;
        a.stride = pr.cg.stride; a.pad = pr.cg.pad; a.OH = pr.OH; a.OW = pr.OW;
    }
    a.alpha_out = alpha_out;
    a.rows_per_slab = rows_per_slab;
    // the plain checksum is one slab summed by one row of blocks; the fused form splits each
    // row block of the tiling over several blocks to have enough loads in flight
    a.rows_per_block = alpha_out ? rows_per_slab : pre_rows_per_block(rows_per_slab, pr.M, pr.K);
    a.beta = beta;
    a.nb = nb;
    a.partial_dots = partial_dots;
    const int subs = a.rows_per_slab / a.rows_per_block;
    dim3 grid((unsigned)pre_grid_x(pr.K, pr.dtype), (unsigned)(cdiv(pr.M, rows_per_slab) * subs)), block(256);
    if (pr.dtype == ABFT_F16) hipLaunchKernelGGL(act_checksum_kernel<DT_F16>, grid, block, 0, st, a);
    else if (pr.dtype == ABFT_BF16) hipLaunchKernelGGL(act_checksum_kernel<DT_BF16>, grid, block, 0, st, a);
    else hipLaunchKernelGGL(act_checksum_kernel<DT_I8>, grid, block, 0, st, a);
    return hipGetLastError();
}

int validate_common(const Problem& pr, int mode, const uint32_t* flag) {
    if (!valid_dtype(pr.dtype)) return ABFT_E_ENUM;
    if (mode < ABFT_NONE || mode > ABFT_GLOBAL_WEIGHTED) return ABFT_E_ENUM;
    if (pr.b_layout != ABFT_B_NK && pr.b_layout != ABFT_B_KN) return ABFT_E_ENUM;
    if (pr.M <= 0 || pr.N <= 0 || pr.K <= 0) return ABFT_E_SHAPE;
    if (!pr.A || !pr.B || !pr.C) return ABFT_E_NULL;
    if (mode != ABFT_NONE && !flag) return ABFT_E_NULL;
    if (!pr.conv && pr.lda < pr.K) return ABFT_E_LD;
    if (pr.b_layout == ABFT_B_NK ? pr.ldb < pr.K : pr.ldb < pr.N) return ABFT_E_LD;
    if (pr.ldc < pr.N) return ABFT_E_LD;
    return ABFT_OK;
}

// Global scheme: where the activation checksum's dot products are formed.  Inside the product
// kernel (direct-to-LDS configurations) it costs about a tenth of the kernel's time; as a
// pass of its own over A it costs a launch plus reading A once.  Take the cheaper by estimate
// (environment variable ABFT_GLOBAL_DOT = fused | pre pins the choice: tuning aid).
bool fused_global(const Problem& pr, const CfgInfo& ci) {
    if (!ci.fast) return false;
    if (ci.kways > 1) return true;  // streaming configurations have no other variant
    static const int force = [] {
        const char* e = std::getenv("ABFT_GLOBAL_DOT");
        return !e ? 0 : (e[0] == 'f' ? 1 : 2);
    }();
    if (force) return force == 1;
    const double t_gemm = 2.0 * pr.M * pr.N * pr.K / (pr.dtype == ABFT_I8 ? 2.0e15 : 1.0e15);
    const double t_pre = 8.0e-6 + (double)pr.M * pr.K * esize(pr.dtype) / 4.5e12;
    // share of the product's time that the in-loop form costs: about a tenth on the 32x32-shape tiles
    // (matrix-unit form, or vector form on 64 x 64 wavefront tiles) and for int8 everywhere; the vector
    // form of fp16 / bf16 on the 16x16-shape tiles: a tenth for fp16 on the 256 x 256 tile, a quarter for
    // bf16 there (three-piece products), a fifth on the smaller tiles (less work per wavefront to hide it in)
    double in_loop = 0.09;
    if (pr.dtype != ABFT_I8 && ci.mi == 16) in_loop = ci.bm == 256 && ci.bn == 256 ? (pr.dtype == ABFT_BF16 ? 0.25 : 0.09) : 0.2;
    return in_loop * t_gemm < t_pre;
}

int run_problem(const Problem& pr, int mode, const void* beta, void* workspace, size_t ws_bytes, uint32_t* flag,
                abft_report_t* report, const abft_fault_t* inject, hipStream_t st) {
    int rc = validate_common(pr, mode, flag);
    if (rc != ABFT_OK) return rc;
    if (mode == ABFT_AUTO) mode = select_mode(pr.M, pr.N, pr.K, pr.dtype);
    // the weighted checks are the global scheme with two more checksum pairs
    const bool weighted = mode == ABFT_GLOBAL_WEIGHTED;
    if (weighted) mode = ABFT_GLOBAL;

    const bool avec = a_vectorisable(pr), bvec = b_vectorisable(pr);
    const bool all16 = avec && bvec;
    const int cfg = pick_cfg(pr.M, pr.N, pr.K, pr.dtype, all16, mode);
    const CfgInfo ci = cfg_info_host(cfg);
    const int bk = ci.bk_bytes / esize(pr.dtype);

    GemmArgs g;
    std::memset(&g, 0, sizeof g);
    g.A = reinterpret_cast<const char*>(pr.A);
    g.B = reinterpret_cast<const char*>(pr.B);
    g.C = reinterpret_cast<char*>(pr.C);
    g.M = pr.M; g.N = pr.N; g.K = pr.K;
    g.lda = pr.lda; g.ldb = pr.ldb; g.ldc = pr.ldc;
    g.b_sn = pr.b_layout == ABFT_B_NK ? pr.ldb : 1;
    g.b_sk = pr.b_layout == ABFT_B_NK ? 1 : pr.ldb;
    g.a_vec = avec; g.b_vec = bvec;
    g.conv = pr.conv ? 1 : 0;
    if (pr.conv) {
        g.imgpitch = pr.imgpitch; g.rowpitch = pr.rowpitch; g.pix = pr.pix;
        g.H = pr.cg.H; g.W = pr.cg.W; g.Cin = pr.cg.Cin; g.KH = pr.cg.KH; g.KW = pr.cg.KW;
        g.stride = pr.cg.stride; g.pad = pr.cg.pad; g.OH = pr.OH; g.OW = pr.OW;
    }
    // (they ride in spare columns of the streaming kernel's extra matrix operand: latency-bound
    // products with fp16 or int8 operands)
    if (weighted && (!cfg_is_stream(cfg) || pr.dtype == ABFT_BF16)) return ABFT_E_UNSUPPORTED;
    g.tiles_m = (int)cdiv(pr.M, ci.bm);
    g.tiles_n = (int)cdiv(pr.N, ci.bn);
    g.flag = flag;
    g.act = pr.act;
    g.report = reinterpret_cast<Report*>(report);
    const int tol_K = pr.tol_K > 0 ? pr.tol_K : pr.K;
    g.tol_coeff = tol_coeff(tol_K, pr.dtype, mode) + tol_half_coeff(pr.dtype, mode, ci.wm, ci.wn, cfg == CFG_G16 ? 16 : 32);
    g.f_row = g.f_col = -1; g.f_bit = 0; g.f_kt = -1;
    // (the streaming kernel stores through an epilogue of its own, the 16-row shapes hold other rows per lane)
    if (pr.alpha_out && pr.dtype != ABFT_I8 && !cfg_is_stream(cfg) && cfg != CFG_G16) {
        g.alpha_out = pr.alpha_out;
        g.ld_alpha_out = pr.ld_alpha_out;
        if (pr.alpha_emitted) *pr.alpha_emitted = true;
    }

    bool inj = false;
    if (inject) {
        if (inject->row < 0 || inject->row >= pr.M || inject->col < 0 || inject->col >= pr.N) return ABFT_E_INJECT;
        if (inject->bit < 0 || inject->bit > 31) return ABFT_E_INJECT;
        if (inject->k_after < -2) return ABFT_E_INJECT;
        if (inject->k_after >= 0) {
            if (inject->k_after == 0 || inject->k_after % bk != 0 || inject->k_after >= pr.K) return ABFT_E_INJECT;
            g.f_kt = inject->k_after / bk - 1;
        }
        // -2: the finished value after the partial tiles of several wavefronts have been added (the
        // streaming configurations); the same as -1 where one wavefront forms the whole sum
        if (inject->k_after == -2 && ci.kways > 1) g.f_kt = -2;
        g.f_row = (int)inject->row; g.f_col = (int)inject->col; g.f_bit = inject->bit;
        inj = true;
    }

    WsLayout w;
    std::memset(&w, 0, sizeof w);
    int kmode = mode;  // the kernels' scheme index
    char* ws = reinterpret_cast<char*>(workspace);
    const void* beta_used = beta;
    if (mode == ABFT_GLOBAL) {
        w = ws_layout(pr.M, pr.N, pr.K, cfg);
        if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < w.total) return ABFT_E_WORKSPACE;
        g.tol_l1 = tol_bias_coeff(tol_K, pr.dtype, mode);
        if (!beta_used) {
            if (launch_weight_checksum(pr.K, pr.N, pr.B, pr.ldb, pr.b_layout, pr.dtype, ci.bn, ws + w.off_beta,
                                       st) != hipSuccess)
                return ABFT_E_HIP;
            beta_used = ws + w.off_beta;
        }
        if (weighted) kmode = MODE_GLOBAL_W;
        // (not on the eight-wavefront 128 x 128 tile: its wavefront tiles are so small that the sums' ring
        // costs more than the in-loop form: 46 against 44.5 us at 1024 x 4096 x 4096)
        if (pr.alpha_in && !weighted && !pr.conv && pr.dtype != ABFT_I8 && ci.fast && ci.kways == 1 && cfg != CFG_F128E) {
            // steps 1-2 were the previous layer's: its epilogue left the column sums of this
            // layer's A per 32-row block; one multiplication per lane and k tile is all that is left
            kmode = MODE_GLOBAL_FED;
            g_handover_launches.fetch_add(1, std::memory_order_relaxed);
            g.alpha_in = pr.alpha_in;
            g.beta_k = reinterpret_cast<const char*>(beta_used) + beta_k_offset(pr.K, g.tiles_n);
        } else if (fused_global(pr, ci)) {
            // the direct-to-LDS kernel forms the activation checksum's dot product with the weight
            // checksums itself, from the A tiles it multiplies (steps 1-3 inside the product's loop)
            g.beta_k = reinterpret_cast<const char*>(beta_used) + beta_k_offset(pr.K, g.tiles_n);
            g.beta_p = reinterpret_cast<const char*>(beta_used) + beta_p_offset(pr.K, g.tiles_n);
            g.beta_r = reinterpret_cast<const char*>(beta_used) + beta_r_offset(pr.K, g.tiles_n);
        } else {
            kmode = MODE_GLOBAL_PRE;
            g.partial_dots = ws + w.off_pd;
            g.n_parts = pre_grid_x(pr.K, pr.dtype) * (ci.bm / pre_rows_per_block(ci.bm, pr.M, pr.K));
            // steps 1-2: activation checksum of every row block of the tiling and its partial dot
            // products with the weight checksums
            if (launch_act_checksum(pr, nullptr, ci.bm, beta_used, g.tiles_n, ws + w.off_pd, st) != hipSuccess)
                return ABFT_E_HIP;
        }
    }

    hipError_t e;
    if (g_ev_start && hipEventRecord(g_ev_start, st) != hipSuccess) return ABFT_E_HIP;
    if (pr.dtype == ABFT_F16) e = launch_gemm_f16(cfg, kmode, inj, g, st);
    else if (pr.dtype == ABFT_BF16) e = launch_gemm_bf16(cfg, kmode, inj, g, st);
    else e = launch_gemm_i8(cfg, kmode, inj, g, st);
    if (e != hipSuccess) return ABFT_E_HIP;
    if (g_ev_stop && hipEventRecord(g_ev_stop, st) != hipSuccess) return ABFT_E_HIP;

    return ABFT_OK;
}

int conv_problem(const abft_conv_t* conv, int N, Problem& pr) {
    if (!conv) return ABFT_E_NULL;
    if (conv->batch <= 0 || conv->H <= 0 || conv->W <= 0 || conv->Cin <= 0 || conv->KH <= 0 || conv->KW <= 0 ||
        conv->stride <= 0 || conv->pad < 0)
        return ABFT_E_SHAPE;
    if (conv->H + 2 * conv->pad < conv->KH || conv->W + 2 * conv->pad < conv->KW) return ABFT_E_SHAPE;
    pr.conv = true;
    pr.cg = *conv;
    pr.OH = conv_out(conv->H, conv->KH, conv->stride, conv->pad);
    pr.OW = conv_out(conv->W, conv->KW, conv->stride, conv->pad);
    long long M = (long long)conv->batch * pr.OH * pr.OW;
    long long K = (long long)conv->KH * conv->KW * conv->Cin;
    if (M <= 0 || M > 0x7fffffffLL || K > 0x7fffffffLL) return ABFT_E_SHAPE;
    pr.M = (int)M;
    pr.K = (int)K;
    pr.N = N;
    pr.lda = pr.K;
    pr.pix = conv->Cin;
    pr.rowpitch = (long long)conv->W * conv->Cin;
    pr.imgpitch = pr.rowpitch * conv->H;
    // a 1 x 1 filter at stride 1 without padding is the plain product on the NHWC tensor read as
    // an M x Cin matrix
    if (conv->KH == 1 && conv->KW == 1 && conv->stride == 1 && conv->pad == 0) {
        pr.conv = false;
        pr.lda = conv->Cin;
    }
    return ABFT_OK;
}

// Lowering of a convolution with few input channels to row segments (see conv_pad_kernel).
struct ConvLowering {
    bool ok;
    int seg, segp, Kp, Hp;
    long long rowp;
    size_t xp_bytes, bp_bytes;
};
ConvLowering conv_lowering(const Problem& pr) {
    ConvLowering lw;
    std::memset(&lw, 0, sizeof lw);
    if (!pr.conv) return lw;
    const abft_conv_t& c = pr.cg;
    const int es = esize(pr.dtype), epc = 16 / es;
    if ((c.Cin * es) % 16 == 0) return lw;                      // chunks already line up with the channels
    if ((long long)c.KW * c.Cin > 64) return lw;                // long runs gain little
    if (((long long)c.stride * c.Cin * es) % 4 != 0) return lw;  // chunk addresses must be 4-byte aligned
    lw.seg = c.KW * c.Cin;
    lw.segp = (int)align_up((size_t)lw.seg, (size_t)epc);
    // whole k tiles of 128 bytes, so that the direct-to-LDS kernel applies (the tail multiplies
    // input rows below the window, or zeros, with zero weights)
    lw.Kp = (int)align_up((size_t)c.KH * lw.segp, (size_t)(128 / es));
    lw.Hp = c.H + 2 * c.pad;
    const long long need = std::max((long long)(c.W + 2 * c.pad) * c.Cin,
                                    (long long)(pr.OW - 1) * c.stride * c.Cin + lw.segp);
    lw.rowp = (long long)align_up((size_t)need, (size_t)epc);
    lw.xp_bytes = align_up((size_t)c.batch * lw.Hp * lw.rowp * es, 256);
    lw.bp_bytes = align_up((size_t)pr.N * lw.Kp * es, 256);
    lw.ok = true;
    return lw;
}

size_t plain_workspace_bytes(int M, int N, int K, int dtype, int mode);

// bytes of workspace that let a convolution run lowered: the lowered product's own scratch, the
// padded input, the re-ordered weights
size_t lowered_workspace_bytes(const Problem& pr, const ConvLowering& lw, int mode) {
    return align_up(plain_workspace_bytes(pr.M, pr.N, lw.Kp, pr.dtype, mode), 256) + lw.xp_bytes + lw.bp_bytes;
}

// Weights of a lowered convolution prepared ahead of the call (a plan does this once, offline:
// the weights are known before inference, Sec. 2.1): the re-ordered N x Kp matrix and, for the
// global scheme, its weight checksums per block of beta_block_n columns.
struct LoweredWeights {
    const void* bp;
    const void* beta;
    int beta_block_n;
};

hipError_t launch_conv_weights(const Problem& pr, const ConvLowering& lw, char* bp, hipStream_t st) {
    const long long sn = pr.b_layout == ABFT_B_NK ? pr.ldb : 1, sk = pr.b_layout == ABFT_B_NK ? 1 : pr.ldb;
    dim3 grid((unsigned)cdiv((long long)pr.N * lw.Kp, 256)), block(256);
    if (esize(pr.dtype) == 2)
        hipLaunchKernelGGL(conv_weights_kernel<2>, grid, block, 0, st, reinterpret_cast<const char*>(pr.B), sn, sk, bp,
                           pr.N, lw.Kp, lw.segp, lw.seg, pr.cg.KH);
    else
        hipLaunchKernelGGL(conv_weights_kernel<1>, grid, block, 0, st, reinterpret_cast<const char*>(pr.B), sn, sk, bp,
                           pr.N, lw.Kp, lw.segp, lw.seg, pr.cg.KH);
    return hipGetLastError();
}

// the lowered product of a convolution: same C, k re-ordered as (filter row, padded run)
Problem lowered_problem(const Problem& pr, const ConvLowering& lw, const void* xp, const void* bp) {
    const abft_conv_t& c = pr.cg;
    Problem q = pr;
    q.A = xp;
    q.B = bp;
    q.b_layout = ABFT_B_NK;
    q.ldb = lw.Kp;
    q.K = lw.Kp;
    q.lda = lw.Kp;
    q.tol_K = pr.K;
    q.cg.H = lw.Hp;
    q.cg.W = (pr.OW - 1) * c.stride + 1;  // every window start lies inside the padded row
    q.cg.Cin = lw.segp;
    q.cg.KW = 1;
    q.cg.pad = 0;
    q.pix = c.Cin;
    q.rowpitch = lw.rowp;
    q.imgpitch = lw.rowp * lw.Hp;
    return q;
}

// a convolution: lowered to row segments when it qualifies and the workspace has the room.
// A fault planted in a running accumulator (k_after >= 0) counts k in the order of abft_conv_t,
// which the lowered product does not keep: such a call runs unlowered.
int run_conv(const Problem& pr, int mode, const void* beta, void* workspace, size_t ws_bytes, uint32_t* flag,
             abft_report_t* report, const abft_fault_t* inject, hipStream_t st, const LoweredWeights* pre = nullptr) {
    const int rc = validate_common(pr, mode, flag);
    if (rc != ABFT_OK) return rc;
    if (mode == ABFT_AUTO) mode = select_mode(pr.M, pr.N, pr.K, pr.dtype);
    const ConvLowering lw = conv_lowering(pr);
    const size_t own_weights = pre ? 0 : lw.bp_bytes;
    if (!lw.ok || (inject && inject->k_after >= 0) || !workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) ||
        ws_bytes < lowered_workspace_bytes(pr, lw, mode) - (lw.bp_bytes - own_weights))
        return run_problem(pr, mode, beta, workspace, ws_bytes, flag, report, inject, st);
    const abft_conv_t& c = pr.cg;
    const int es = esize(pr.dtype);
    const size_t inner = align_up(plain_workspace_bytes(pr.M, pr.N, lw.Kp, pr.dtype, mode), 256);
    char* xp = reinterpret_cast<char*>(workspace) + inner;
    char* bp = xp + lw.xp_bytes;
    {
        const long long chunks_per_row = lw.rowp / (16 / es);
        const long long total = (long long)c.batch * lw.Hp * chunks_per_row;
        dim3 grid((unsigned)cdiv(total, 256)), block(256);
        if (es == 2)
            hipLaunchKernelGGL(conv_pad_kernel<2>, grid, block, 0, st, reinterpret_cast<const char*>(pr.A), xp, c.H,
                               c.W * c.Cin, c.pad, c.pad * c.Cin, lw.Hp, lw.rowp, chunks_per_row, total);
        else
            hipLaunchKernelGGL(conv_pad_kernel<1>, grid, block, 0, st, reinterpret_cast<const char*>(pr.A), xp, c.H,
                               c.W * c.Cin, c.pad, c.pad * c.Cin, lw.Hp, lw.rowp, chunks_per_row, total);
        if (hipGetLastError() != hipSuccess) return ABFT_E_HIP;
        if (!pre && launch_conv_weights(pr, lw, bp, st) != hipSuccess) return ABFT_E_HIP;
    }
    const Problem q = lowered_problem(pr, lw, xp, pre ? pre->bp : bp);
    // offline weight checksums of the lowered weights fit only the tiling they were made for
    const void* qbeta = nullptr;
    if (pre && pre->beta && mode == ABFT_GLOBAL) {
        const int bn_now = cfg_info_host(pick_cfg(q.M, q.N, q.K, q.dtype, a_vectorisable(q) && b_vectorisable(q), ABFT_GLOBAL)).bn;
        if (bn_now == pre->beta_block_n) qbeta = pre->beta;
    }
    return run_problem(q, mode, qbeta, workspace, inner, flag, report, inject, st);
}

size_t plain_workspace_bytes(int M, int N, int K, int dtype, int mode) {
    if (mode == ABFT_AUTO) mode = select_mode(M, N, K, dtype);
    // only the global scheme keeps anything outside the operands
    return (mode == ABFT_GLOBAL || mode == ABFT_GLOBAL_WEIGHTED) ? ws_bytes_any_cfg(M, N, K) : 0;
}

}  // namespace

// ------------------------------------------------------------------------- //
// plans
// ------------------------------------------------------------------------- //
struct abft_plan {
    struct Layer {
        abft_layer_t desc;
        int mode;
        void* beta;       // per-column-block weight checksums, blocks of beta_block_n columns
        int beta_block_n;
        void* workspace;
        size_t ws_bytes;
        double t_us[3];
        int act;          // abft_act_t applied to the stored output
        // a convolution that runs lowered to row segments: its re-ordered weights and their
        // checksums, made once at creation
        void* lowered_B;
        void* lowered_beta;
        int lowered_block_n;
        // a fully-connected layer that can run inside a chain of layers in one launch
        // (abft_plan_run_chain): weight checksums per block of 32 columns, its tiling there
        void* chain_beta;
        // activation checksums of this layer's input, left by the layer before it in a chain run
        // layer by layer: ceil(M / 32) x K floats (fully-connected fp16 / bf16 layers)
        float* alpha32;
        // diagnostics block and planted fault (test hook) handed to every run of the layer
        abft_report_t* report;
        abft_fault_t fault;
        bool has_fault;
    };
    std::vector<Layer> layers;
    // completion flags and status word of the chain kernel (zero at creation; see mlp_chain.h)
    unsigned* chain_flags = nullptr;
    int chain_spin_limit = 1 << 20;

};

namespace {

// Can this layer run inside the chain kernel?  Fully connected, fp16 / bf16, weights with k
// contiguous and 16-byte aligned rows, K whole k tiles of 128 bytes.
bool chain_layer_ok(const abft_layer_t& d) {
    if (d.has_conv || d.dtype == ABFT_I8 || d.b_layout != ABFT_B_NK) return false;
    return ((long long)d.K * 2) % 128 == 0 && (d.ldb * 2) % 16 == 0 && aligned16(d.B);
}

}  // namespace

// ------------------------------------------------------------------------- //
// exported functions
// ------------------------------------------------------------------------- //
extern "C" {

int abft_gemm(int M, int N, int K, const void* A, int64_t lda, const void* B, int64_t ldb, int b_layout, void* C,
              int64_t ldc, int dtype, int mode, const void* beta, void* workspace, size_t workspace_bytes,
              uint32_t* fault_flag, abft_report_t* report, const abft_fault_t* inject, void* stream) {
    Problem pr;
    std::memset(&pr, 0, sizeof pr);
    pr.M = M; pr.N = N; pr.K = K; pr.dtype = dtype; pr.b_layout = b_layout;
    pr.A = A; pr.lda = lda; pr.B = B; pr.ldb = ldb; pr.C = C; pr.ldc = ldc;
    pr.conv = false;
    return run_problem(pr, mode, beta, workspace, workspace_bytes, fault_flag, report, inject,
                       reinterpret_cast<hipStream_t>(stream));
}

int abft_gemm_static(int M, int N, int K, const void* A, int64_t lda, const void* B, int64_t ldb, int b_layout,
                     void* C, int64_t ldc, int dtype, int mode, const void* beta, uint32_t* fault_flag,
                     abft_report_t* report, const abft_fault_t* inject, void* stream) {
    Problem pr;
    std::memset(&pr, 0, sizeof pr);
    pr.M = M; pr.N = N; pr.K = K; pr.dtype = dtype; pr.b_layout = b_layout;
    pr.A = A; pr.lda = lda; pr.B = B; pr.ldb = ldb; pr.C = C; pr.ldc = ldc;
    pr.conv = false;
    void* scratch = scratch_of_current_device();
    if (!scratch) return ABFT_E_HIP;
    // (a product whose scratch does not fit comes back as ABFT_E_WORKSPACE before anything is launched)
    return run_problem(pr, mode, beta, scratch, STATIC_SCRATCH_BYTES, fault_flag, report, inject,
                       reinterpret_cast<hipStream_t>(stream));
}

size_t abft_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int abft_conv(const abft_conv_t* conv, int N, const void* x, const void* B, int64_t ldb, int b_layout, void* C,
              int64_t ldc, int dtype, int mode, const void* beta, void* workspace, size_t workspace_bytes,
              uint32_t* fault_flag, abft_report_t* report, const abft_fault_t* inject, void* stream) {
    Problem pr;
    std::memset(&pr, 0, sizeof pr);
    if (N <= 0) return ABFT_E_SHAPE;
    int rc = conv_problem(conv, N, pr);
    if (rc != ABFT_OK) return rc;
    pr.dtype = dtype; pr.b_layout = b_layout;
    pr.A = x; pr.B = B; pr.ldb = ldb; pr.C = C; pr.ldc = ldc;
    return run_conv(pr, mode, beta, workspace, workspace_bytes, fault_flag, report, inject,
                    reinterpret_cast<hipStream_t>(stream));
}

size_t abft_workspace_bytes(int M, int N, int K, int dtype, int mode) {
    if (M <= 0 || N <= 0 || K <= 0 || !valid_dtype(dtype)) return 0;
    return plain_workspace_bytes(M, N, K, dtype, mode);
}

size_t abft_conv_workspace_bytes(const abft_conv_t* conv, int N, int dtype, int mode) {
    Problem pr;
    std::memset(&pr, 0, sizeof pr);
    if (N <= 0 || !valid_dtype(dtype) || conv_problem(conv, N, pr) != ABFT_OK) return 0;
    pr.dtype = dtype;
    if (mode == ABFT_AUTO) mode = select_mode(pr.M, pr.N, pr.K, dtype);
    const ConvLowering lw = conv_lowering(pr);
    const size_t plain = plain_workspace_bytes(pr.M, pr.N, pr.K, dtype, mode);
    return lw.ok ? std::max(plain, lowered_workspace_bytes(pr, lw, mode)) : plain;
}

size_t abft_beta_bytes(int K, int N, int block_n) {
    if (K <= 0 || N <= 0) return 0;
    if (block_n <= 0 || block_n > N) block_n = N;
    return beta_total_bytes(K, (int)cdiv(N, block_n));
}

int abft_weight_checksum(int K, int N, const void* B, int64_t ldb, int b_layout, int dtype, int block_n,
                         void* beta, void* stream) {
    if (!valid_dtype(dtype)) return ABFT_E_ENUM;
    if (b_layout != ABFT_B_NK && b_layout != ABFT_B_KN) return ABFT_E_ENUM;
    if (K <= 0 || N <= 0) return ABFT_E_SHAPE;
    if (!B || !beta) return ABFT_E_NULL;
    if (b_layout == ABFT_B_NK ? ldb < K : ldb < N) return ABFT_E_LD;
    return launch_weight_checksum(K, N, B, ldb, b_layout, dtype, block_n, beta,
                                  reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? ABFT_OK
               : ABFT_E_HIP;
}

int abft_activation_checksum(int M, int K, const void* A, int64_t lda, const abft_conv_t* conv, int dtype,
                             void* alpha, void* stream) {
    if (!valid_dtype(dtype)) return ABFT_E_ENUM;
    if (!A || !alpha) return ABFT_E_NULL;
    Problem pr;
    std::memset(&pr, 0, sizeof pr);
    pr.dtype = dtype;
    if (conv) {
        int rc = conv_problem(conv, 1, pr);
        if (rc != ABFT_OK) return rc;
        if (pr.M != M || pr.K != K) return ABFT_E_SHAPE;
    } else {
        if (M <= 0 || K <= 0) return ABFT_E_SHAPE;
        if (lda < K) return ABFT_E_LD;
        pr.M = M; pr.K = K; pr.lda = lda;
    }
    pr.A = A;
    // one slab covering every row: the plain 1 x K checksum
    return launch_act_checksum(pr, alpha, M, nullptr, 0, nullptr, reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? ABFT_OK
               : ABFT_E_HIP;
}

int abft_k_ways(int M, int N, int K, int dtype, int aligned, int mode, int* ways, int* step) {
    if (!valid_dtype(dtype)) return ABFT_E_ENUM;
    if (M <= 0 || N <= 0 || K <= 0) return ABFT_E_SHAPE;
    if (mode == ABFT_AUTO) mode = select_mode(M, N, K, dtype);
    const CfgInfo ci = cfg_info_host(pick_cfg(M, N, K, dtype, aligned != 0, mode));
    if (ways) *ways = ci.kways;
    if (step) *step = ci.kway_bytes / esize(dtype);
    return ABFT_OK;
}

double abft_arithmetic_intensity(int M, int N, int K, int dtype) {
    if (M <= 0 || N <= 0 || K <= 0 || !valid_dtype(dtype)) return 0.0;
    return intensity(M, N, K, dtype);
}

double abft_cmr(int dtype) { return valid_dtype(dtype) ? cmr_of(dtype) : 0.0; }

void abft_set_cmr(int dtype, double value) {
    if (valid_dtype(dtype)) g_cmr_override[dtype] = value > 0.0 ? value : 0.0;
}

int abft_select(int M, int N, int K, int dtype) {
    if (!valid_dtype(dtype)) return ABFT_E_ENUM;
    if (M <= 0 || N <= 0 || K <= 0) return ABFT_E_SHAPE;
    return select_mode(M, N, K, dtype);
}

int abft_tile_shape(int M, int N, int K, int dtype, int aligned, int* tile_m, int* tile_n, int* k_step) {
    if (!valid_dtype(dtype)) return ABFT_E_ENUM;
    if (M <= 0 || N <= 0 || K <= 0) return ABFT_E_SHAPE;
    CfgInfo ci = cfg_info_host(pick_cfg(M, N, K, dtype, aligned != 0, ABFT_THREAD));
    if (tile_m) *tile_m = ci.wm;
    if (tile_n) *tile_n = ci.wn;
    if (k_step) *k_step = ci.bk_bytes / esize(dtype);
    return ABFT_OK;
}

int abft_region_shape(int M, int N, int K, int dtype, int aligned, int* region_m, int* region_n) {
    if (!valid_dtype(dtype)) return ABFT_E_ENUM;
    if (M <= 0 || N <= 0 || K <= 0) return ABFT_E_SHAPE;
    CfgInfo ci = cfg_info_host(pick_cfg(M, N, K, dtype, aligned != 0, ABFT_GLOBAL));
    if (region_m) *region_m = ci.bm;
    if (region_n) *region_n = ci.bn;
    return ABFT_OK;
}

double abft_tolerance_coeff(int K, int dtype, int mode) {
    if (!valid_dtype(dtype) || K <= 0) return 0.0;
    return tol_coeff(K, dtype, mode);
}

double abft_tolerance_half_coeff(int dtype, int mode, int tile_m, int tile_n) {
    if (!valid_dtype(dtype) || tile_m <= 0 || tile_n <= 0) return 0.0;
    return tol_half_coeff(dtype, mode, tile_m, tile_n, tile_m < 32 ? 16 : 32);
}

double abft_tolerance_bias_coeff(int K, int dtype, int mode) {
    if (!valid_dtype(dtype) || K <= 0) return 0.0;
    return tol_bias_coeff(K, dtype, mode);
}

int abft_plan_create(abft_plan_t** plan, const abft_layer_t* layers, int n_layers, int profile, void* stream) {
    if (!plan || !layers) return ABFT_E_NULL;
    if (n_layers <= 0) return ABFT_E_SHAPE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    abft_plan* p = new (std::nothrow) abft_plan;
    if (!p) return ABFT_E_HIP;
    int rc = ABFT_OK;
    for (int i = 0; i < n_layers && rc == ABFT_OK; ++i) {
        abft_plan::Layer L;
        std::memset(&L, 0, sizeof L);
        L.desc = layers[i];
        const abft_layer_t& d = L.desc;
        if (!valid_dtype(d.dtype)) { rc = ABFT_E_ENUM; break; }
        if (d.b_layout != ABFT_B_NK && d.b_layout != ABFT_B_KN) { rc = ABFT_E_ENUM; break; }
        if (d.M <= 0 || d.N <= 0 || d.K <= 0) { rc = ABFT_E_SHAPE; break; }
        if (!d.B) { rc = ABFT_E_NULL; break; }
        if (d.has_conv) {
            Problem pr;
            std::memset(&pr, 0, sizeof pr);
            rc = conv_problem(&d.conv, d.N, pr);
            if (rc != ABFT_OK) break;
            if (pr.M != d.M || pr.K != d.K) { rc = ABFT_E_SHAPE; break; }
        }
        L.mode = select_mode(d.M, d.N, d.K, d.dtype);
        // offline weight checksum and workspace for the global scheme (kept for either
        // choice so that profiling can time both)
        L.ws_bytes = ws_bytes_any_cfg(d.M, d.N, d.K);
        for (int md = ABFT_NONE; md <= ABFT_THREAD; ++md) {
            const size_t need = d.has_conv ? abft_conv_workspace_bytes(&d.conv, d.N, d.dtype, md)
                                           : abft_workspace_bytes(d.M, d.N, d.K, d.dtype, md);
            if (need > L.ws_bytes) L.ws_bytes = need;
        }
        {
            // the tiling the layer will run with when its activations are 16-byte aligned
            const int es = esize(d.dtype);
            const bool b16 = d.b_layout == ABFT_B_NK && aligned16(d.B) && (d.K * es) % 16 == 0 && (d.ldb * es) % 16 == 0;
            const bool a16 = d.has_conv ? (d.conv.Cin * es) % 16 == 0 : (d.K * es) % 16 == 0;
            L.beta_block_n = cfg_info_host(pick_cfg(d.M, d.N, d.K, d.dtype, a16 && b16, ABFT_GLOBAL)).bn;
        }
        if (hipMalloc(&L.beta, beta_total_bytes(d.K, (int)cdiv(d.N, L.beta_block_n))) != hipSuccess) { rc = ABFT_E_HIP; break; }
        if (hipMalloc(&L.workspace, L.ws_bytes) != hipSuccess) { (void)hipFree(L.beta); rc = ABFT_E_HIP; break; }
        p->layers.push_back(L);
        if (d.dtype != ABFT_I8 && (!d.has_conv || (d.conv.KH == 1 && d.conv.KW == 1 && d.conv.stride == 1 && d.conv.pad == 0))) {
            // (a layer that reads a plain M x K matrix can take its activation checksums from the layer before)
            abft_plan::Layer& PL = p->layers.back();
            if (hipMalloc(reinterpret_cast<void**>(&PL.alpha32), (size_t)cdiv(d.M, 32) * d.K * sizeof(float)) != hipSuccess) {
                rc = ABFT_E_HIP;
                break;
            }
        }
        if (chain_layer_ok(d)) {
            abft_plan::Layer& PL = p->layers.back();
            if (hipMalloc(&PL.chain_beta, beta_total_bytes(d.K, (int)cdiv(d.N, 32))) != hipSuccess ||
                launch_weight_checksum(d.K, d.N, d.B, d.ldb, d.b_layout, d.dtype, 32, PL.chain_beta, st) != hipSuccess) {
                rc = ABFT_E_HIP;
                break;
            }
        }
        if (d.has_conv) {
            // few input channels: the layer will run lowered to row segments; its weights are
            // re-ordered, and their checksums formed, here and now (offline, Sec. 2.5)
            Problem pr;
            std::memset(&pr, 0, sizeof pr);
            (void)conv_problem(&d.conv, d.N, pr);
            pr.dtype = d.dtype; pr.b_layout = d.b_layout; pr.B = d.B; pr.ldb = d.ldb;
            const ConvLowering lw = conv_lowering(pr);
            if (lw.ok) {
                abft_plan::Layer& PL = p->layers.back();
                PL.lowered_block_n = cfg_info_host(pick_cfg(d.M, d.N, lw.Kp, d.dtype, true, ABFT_GLOBAL)).bn;
                if (hipMalloc(&PL.lowered_B, lw.bp_bytes) != hipSuccess ||
                    hipMalloc(&PL.lowered_beta, beta_total_bytes(lw.Kp, (int)cdiv(d.N, PL.lowered_block_n))) != hipSuccess ||
                    launch_conv_weights(pr, lw, reinterpret_cast<char*>(PL.lowered_B), st) != hipSuccess ||
                    launch_weight_checksum(lw.Kp, d.N, PL.lowered_B, lw.Kp, ABFT_B_NK, d.dtype, PL.lowered_block_n,
                                           PL.lowered_beta, st) != hipSuccess) {
                    rc = ABFT_E_HIP;
                    break;
                }
            }
        }
        if (launch_weight_checksum(d.K, d.N, d.B, d.ldb, d.b_layout, d.dtype, L.beta_block_n, L.beta, st) !=
            hipSuccess) {
            rc = ABFT_E_HIP;
            break;
        }
    }
    if (rc == ABFT_OK) {
        const size_t bytes = (size_t)(CHAIN_FLAG_WORDS + 64) * sizeof(unsigned);
        if (hipMalloc(reinterpret_cast<void**>(&p->chain_flags), bytes) != hipSuccess ||
            hipMemsetAsync(p->chain_flags, 0, bytes, st) != hipSuccess)
            rc = ABFT_E_HIP;
    }
    if (rc == ABFT_OK && profile) {
        // pre-deployment profiling (Sec. 5.3): time each scheme on scratch inputs, keep the faster
        hipEvent_t e0, e1;
        uint32_t* d_flag = nullptr;
        if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess ||
            hipMalloc(&d_flag, 4) != hipSuccess)
            rc = ABFT_E_HIP;
        for (size_t i = 0; i < p->layers.size() && rc == ABFT_OK; ++i) {
            abft_plan::Layer& L = p->layers[i];
            const abft_layer_t& d = L.desc;
            size_t a_elems = d.has_conv ? (size_t)d.conv.batch * d.conv.H * d.conv.W * d.conv.Cin
                                        : (size_t)d.M * d.K;
            void *A = nullptr, *C = nullptr;
            if (hipMalloc(&A, a_elems * esize(d.dtype)) != hipSuccess) { rc = ABFT_E_HIP; break; }
            if (hipMalloc(&C, (size_t)d.M * d.N * csize(d.dtype)) != hipSuccess) { (void)hipFree(A); rc = ABFT_E_HIP; break; }
            (void)hipMemsetAsync(A, 0, a_elems * esize(d.dtype), st);
            (void)hipMemsetAsync(d_flag, 0, 4, st);
            const int modes[3] = {ABFT_NONE, ABFT_GLOBAL, ABFT_THREAD};
            for (int mi = 0; mi < 3 && rc == ABFT_OK; ++mi) {
                const int reps = 20;
                for (int r = -3; r < reps && rc == ABFT_OK; ++r) {
                    if (r == 0) (void)hipEventRecord(e0, st);
                    int saved = L.mode;
                    L.mode = modes[mi];
                    rc = abft_plan_run(p, (int)i, A, d.K, C, d.N, d_flag, stream);
                    L.mode = saved;
                }
                (void)hipEventRecord(e1, st);
                if (hipEventSynchronize(e1) != hipSuccess) rc = ABFT_E_HIP;
                float ms = 0.f;
                (void)hipEventElapsedTime(&ms, e0, e1);
                L.t_us[mi] = 1000.0 * ms / reps;
            }
            if (rc == ABFT_OK) L.mode = L.t_us[1] <= L.t_us[2] ? ABFT_GLOBAL : ABFT_THREAD;
            (void)hipFree(A);
            (void)hipFree(C);
        }
        if (d_flag) (void)hipFree(d_flag);
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
    }
    if (rc != ABFT_OK) {
        abft_plan_destroy(p);
        return rc;
    }
    *plan = p;
    return ABFT_OK;
}

}  // extern "C"

namespace {

// Does layer `next` of the plan, reading the M x K matrix at (a_next, lda_next) that layer `next - 1`
// is about to store, want that layer's epilogue to leave the column sums of what it stores?  Under
// the global scheme, same M, dtype and K = the producer's N, and when it will run on the kernel that
// takes them.  Returns where they go (the consumer's buffer), or null.
float* handover_target(const abft_plan_t* plan, int next, const void* a_next, int64_t lda_next) {
    const abft_plan::Layer& nx = plan->layers[next];
    const abft_layer_t& d = plan->layers[next - 1].desc;
    const abft_layer_t& e = nx.desc;
    if (nx.mode != ABFT_GLOBAL || !nx.alpha32 || e.M != d.M || e.K != d.N || e.dtype != d.dtype) return nullptr;
    const int es = esize(e.dtype);
    const bool a16 = aligned16(a_next) && (lda_next * es) % 16 == 0 && (e.K * es) % 16 == 0;
    const bool b16 = e.b_layout == ABFT_B_NK && aligned16(e.B) && (e.K * es) % 16 == 0 && (e.ldb * es) % 16 == 0;
    const int cfg = pick_cfg(e.M, e.N, e.K, e.dtype, a16 && b16, ABFT_GLOBAL);
    const CfgInfo ci = cfg_info_host(cfg);
    return (ci.fast && ci.kways == 1 && cfg != CFG_F128E) ? nx.alpha32 : nullptr;
}

// One layer of a plan.  alpha_out (may be null): where to leave the activation checksums of the
// layer that follows (leading dimension ld_alpha_out), *alpha_emitted set when the kernel that ran
// could; alpha_in (may be null): those the layer before left for this layer's input.
int plan_run_layer(abft_plan_t* plan, int layer, const void* A, int64_t lda, void* C, int64_t ldc, uint32_t* fault_flag,
                   void* stream, float* alpha_out, long long ld_alpha_out, bool* alpha_emitted, const float* alpha_in) {
    abft_plan::Layer& L = plan->layers[layer];
    const abft_layer_t& d = L.desc;
    Problem pr;
    std::memset(&pr, 0, sizeof pr);
    if (d.has_conv) {
        int rc = conv_problem(&d.conv, d.N, pr);
        if (rc != ABFT_OK) return rc;
    } else {
        pr.M = d.M; pr.N = d.N; pr.K = d.K; pr.lda = lda;
    }
    pr.dtype = d.dtype; pr.b_layout = d.b_layout;
    pr.A = A; pr.B = d.B; pr.ldb = d.ldb; pr.C = C; pr.ldc = ldc;
    pr.act = L.act;
    pr.alpha_out = alpha_out; pr.ld_alpha_out = ld_alpha_out; pr.alpha_emitted = alpha_emitted; pr.alpha_in = alpha_in;
    // the offline checksums fit the tiling chosen for aligned activations; an input that
    // forces another tiling gets them recomputed into the workspace
    const int bn_now = cfg_info_host(pick_cfg(pr.M, pr.N, pr.K, pr.dtype, a_vectorisable(pr) && b_vectorisable(pr), ABFT_GLOBAL)).bn;
    const void* beta = bn_now == L.beta_block_n ? L.beta : nullptr;
    const abft_fault_t* fault = L.has_fault ? &L.fault : nullptr;
    if (pr.conv) {
        const LoweredWeights pre = {L.lowered_B, L.lowered_beta, L.lowered_block_n};
        return run_conv(pr, L.mode, beta, L.workspace, L.ws_bytes, fault_flag, L.report, fault,
                        reinterpret_cast<hipStream_t>(stream), L.lowered_B ? &pre : nullptr);
    }
    return run_problem(pr, L.mode, beta, L.workspace, L.ws_bytes, fault_flag, L.report, fault,
                       reinterpret_cast<hipStream_t>(stream));
}

}  // namespace

extern "C" {

int abft_plan_run(abft_plan_t* plan, int layer, const void* A, int64_t lda, void* C, int64_t ldc,
                  uint32_t* fault_flag, void* stream) {
    if (!plan || layer < 0 || layer >= (int)plan->layers.size()) return ABFT_E_PLAN;
    return plan_run_layer(plan, layer, A, lda, C, ldc, fault_flag, stream, nullptr, 0, nullptr, nullptr);
}

int abft_plan_run_all(abft_plan_t* plan, const void* const* A, const int64_t* lda, void* const* C,
                      const int64_t* ldc, uint32_t* fault_flag, int event_layer, void* stream) {
    if (!plan) return ABFT_E_PLAN;
    if (!A || !lda || !C || !ldc) return ABFT_E_NULL;
    const hipEvent_t ev0 = g_ev_start, ev1 = g_ev_stop;
    int rc = ABFT_OK;
    const int n = (int)plan->layers.size();
    const float* alpha_in = nullptr;
    for (int i = 0; i < n && rc == ABFT_OK; ++i) {
        // the measurement hook, if set, brackets the product kernel of one layer only
        g_ev_start = i == event_layer ? ev0 : nullptr;
        g_ev_stop = i == event_layer ? ev1 : nullptr;
        // a layer whose input IS the output of the layer before it (same pointer and leading
        // dimension) is chained to it: it can take its activation checksums from that layer's epilogue
        const bool next_chained = i + 1 < n && A[i + 1] == C[i] && lda[i + 1] == ldc[i];
        float* alpha_out = next_chained ? handover_target(plan, i + 1, C[i], ldc[i]) : nullptr;
        bool emitted = false;
        rc = plan_run_layer(plan, i, A[i], lda[i], C[i], ldc[i], fault_flag, stream, alpha_out,
                            alpha_out ? plan->layers[i + 1].desc.K : 0, &emitted, alpha_in);
        alpha_in = emitted ? alpha_out : nullptr;
    }
    g_ev_start = ev0;
    g_ev_stop = ev1;
    return rc;
}

int abft_plan_run_chain(abft_plan_t* plan, int first, int count, const void* A, int64_t lda, void* const* C,
                        const int64_t* ldc, uint32_t* fault_flag, void* stream) {
    if (!plan || first < 0 || count <= 0 || first + count > (int)plan->layers.size()) return ABFT_E_PLAN;
    if (!A || !C || !ldc) return ABFT_E_NULL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // one launch for the whole chain when every layer qualifies; else layer by layer
    bool one_launch = count <= CHAIN_MAX_LAYERS && plan->chain_flags != nullptr;
    const abft_layer_t& d0 = plan->layers[first].desc;
    bool any_check = false;
    for (int i = 0; i < count && one_launch; ++i) {
        const abft_plan::Layer& L = plan->layers[first + i];
        const abft_layer_t& d = L.desc;
        const void* a_i = i == 0 ? A : C[i - 1];
        const int64_t lda_i = i == 0 ? lda : ldc[i - 1];
        // (layers small enough that a launch of their own would run on 32 x 32 tiles too)
        one_launch = L.chain_beta != nullptr && d.dtype == d0.dtype && d.M == d0.M &&
                     pick_cfg(d.M, d.N, d.K, d.dtype, true, L.mode) == CFG_S32 && !L.report && !L.has_fault &&
                     (L.mode == ABFT_NONE || L.mode == ABFT_GLOBAL || L.mode == ABFT_THREAD) && C[i] != nullptr &&
                     aligned16(a_i) && (lda_i * 2) % 16 == 0 && lda_i >= d.K && ldc[i] >= d.N &&
                     (i == 0 || d.K == plan->layers[first + i - 1].desc.N);
        any_check = any_check || L.mode != ABFT_NONE;
    }
    if (one_launch && any_check && !fault_flag) return ABFT_E_NULL;
    if (!one_launch) {
        // Layer by layer.  A layer under the global scheme takes its activation checksums from the
        // epilogue of the layer before it (Sec. 2.4 step 4) when it reads that layer's output as a
        // plain matrix and both run kernels that can do their part; else it forms them itself.
        int rc = ABFT_OK;
        const float* alpha_in = nullptr;
        for (int i = 0; i < count && rc == ABFT_OK; ++i) {
            float* alpha_out = i + 1 < count ? handover_target(plan, first + i + 1, C[i], ldc[i]) : nullptr;
            const long long ld_alpha = alpha_out ? plan->layers[first + i + 1].desc.K : 0;
            bool emitted = false;
            rc = plan_run_layer(plan, first + i, i == 0 ? A : C[i - 1], i == 0 ? lda : ldc[i - 1], C[i], ldc[i], fault_flag,
                                stream, alpha_out, ld_alpha, &emitted, alpha_in);
            alpha_in = emitted ? alpha_out : nullptr;
        }
        return rc;
    }
    ChainArgs a;
    std::memset(&a, 0, sizeof a);
    a.n_layers = count;
    a.M = d0.M;
    a.flags = plan->chain_flags;
    a.status = plan->chain_flags + CHAIN_FLAG_WORDS;
    a.fault_flag = fault_flag ? fault_flag : plan->chain_flags + CHAIN_FLAG_WORDS + 1;   // (unprotected chain: a word of the plan's own)
    a.spin_limit = plan->chain_spin_limit;
    for (int i = 0; i < count; ++i) {
        const abft_plan::Layer& L = plan->layers[first + i];
        const abft_layer_t& d = L.desc;
        ChainLayer& c = a.layer[i];
        c.A = reinterpret_cast<const char*>(i == 0 ? A : C[i - 1]);
        c.lda = i == 0 ? lda : ldc[i - 1];
        c.B = reinterpret_cast<const char*>(d.B);
        c.ldb = d.ldb;
        c.C = reinterpret_cast<char*>(C[i]);
        c.ldc = ldc[i];
        c.N = d.N;
        c.K = d.K;
        const int nb = (int)cdiv(d.N, 32);
        c.beta_k = reinterpret_cast<const char*>(L.chain_beta) + beta_k_offset(d.K, nb);
        c.beta_p = reinterpret_cast<const char*>(L.chain_beta) + beta_p_offset(d.K, nb);
        c.mode = L.mode;          // ABFT_NONE / GLOBAL / THREAD carry the kernels' own numbers
        c.act = L.act;
        c.depends = i > 0;
        c.tol_coeff = tol_coeff(d.K, d.dtype, L.mode);
        c.tol_l1 = tol_bias_coeff(d.K, d.dtype, L.mode);
    }
    const hipError_t e = d0.dtype == ABFT_F16 ? launch_mlp_chain_f16(a, st) : launch_mlp_chain_bf16(a, st);
    return e == hipSuccess ? ABFT_OK : ABFT_E_HIP;
}

int abft_plan_chain_status(abft_plan_t* plan, uint32_t* status, void* stream) {
    if (!plan || !plan->chain_flags) return ABFT_E_PLAN;
    if (!status) return ABFT_E_NULL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(status, plan->chain_flags + CHAIN_FLAG_WORDS, sizeof(uint32_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return ABFT_E_HIP;
    return ABFT_OK;
}

int abft_plan_chain_reset(abft_plan_t* plan, int spin_limit, void* stream) {
    if (!plan || !plan->chain_flags) return ABFT_E_PLAN;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (hipMemsetAsync(plan->chain_flags, 0, (size_t)(CHAIN_FLAG_WORDS + 64) * sizeof(unsigned), st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return ABFT_E_HIP;
    plan->chain_spin_limit = spin_limit >= 0 ? spin_limit : (1 << 20);
    return ABFT_OK;
}

long long abft_handover_launches(void) { return g_handover_launches.load(std::memory_order_relaxed); }

int abft_plan_set_diagnostics(abft_plan_t* plan, int layer, abft_report_t* report, const abft_fault_t* inject) {
    if (!plan || layer < 0 || layer >= (int)plan->layers.size()) return ABFT_E_PLAN;
    abft_plan::Layer& L = plan->layers[layer];
    L.report = report;
    L.has_fault = inject != nullptr;
    if (inject) L.fault = *inject;
    return ABFT_OK;
}

int abft_plan_set_mode(abft_plan_t* plan, int layer, int mode) {
    if (!plan || layer < 0 || layer >= (int)plan->layers.size()) return ABFT_E_PLAN;
    if (mode < ABFT_NONE || mode > ABFT_GLOBAL_WEIGHTED) return ABFT_E_ENUM;
    abft_plan::Layer& L = plan->layers[layer];
    L.mode = mode == ABFT_AUTO ? select_mode(L.desc.M, L.desc.N, L.desc.K, L.desc.dtype) : mode;
    return ABFT_OK;
}

int abft_plan_set_activation(abft_plan_t* plan, int layer, int act) {
    if (!plan || layer < 0 || layer >= (int)plan->layers.size()) return ABFT_E_PLAN;
    if (act != ABFT_ACT_NONE && act != ABFT_ACT_RELU) return ABFT_E_ENUM;
    plan->layers[layer].act = act;
    return ABFT_OK;
}

int abft_plan_activation(const abft_plan_t* plan, int layer) {
    if (!plan || layer < 0 || layer >= (int)plan->layers.size()) return ABFT_E_PLAN;
    return plan->layers[layer].act;
}

int abft_plan_mode(const abft_plan_t* plan, int layer) {
    if (!plan || layer < 0 || layer >= (int)plan->layers.size()) return ABFT_E_PLAN;
    return plan->layers[layer].mode;
}

int abft_plan_times(const abft_plan_t* plan, int layer, double* out3) {
    if (!plan || layer < 0 || layer >= (int)plan->layers.size()) return ABFT_E_PLAN;
    if (!out3) return ABFT_E_NULL;
    for (int i = 0; i < 3; ++i) out3[i] = plan->layers[layer].t_us[i];
    return ABFT_OK;
}

void abft_plan_destroy(abft_plan_t* plan) {
    if (!plan) return;
    for (auto& L : plan->layers) {
        if (L.beta) (void)hipFree(L.beta);
        if (L.workspace) (void)hipFree(L.workspace);
        if (L.lowered_B) (void)hipFree(L.lowered_B);
        if (L.lowered_beta) (void)hipFree(L.lowered_beta);
        if (L.chain_beta) (void)hipFree(L.chain_beta);
        if (L.alpha32) (void)hipFree(L.alpha32);
    }
    if (plan->chain_flags) (void)hipFree(plan->chain_flags);
    delete plan;
}

const char* abft_strerror(int code) {
    switch (code) {
        case ABFT_OK: return "ok";
        case ABFT_E_NULL: return "a required pointer is NULL";
        case ABFT_E_SHAPE: return "bad problem shape";
        case ABFT_E_LD: return "leading dimension smaller than the row length";
        case ABFT_E_ENUM: return "unknown dtype, mode or layout";
        case ABFT_E_WORKSPACE: return "workspace missing, misaligned or too small";
        case ABFT_E_INJECT: return "fault descriptor out of range";
        case ABFT_E_HIP: return "HIP runtime call failed";
        case ABFT_E_PLAN: return "bad plan handle or layer index";
        case ABFT_E_UNSUPPORTED: return "scheme not available for this product";
    }
    return "unknown error code";
}

int abft_version(void) { return 100; }

}  // extern "C"

namespace {
// MFMAs from registers only: each wavefront keeps the fragments of a 128 x 64 register tile
// (TM + TN fragments of 16 bytes per lane) and multiplies them `iters` times into its TM x TN
// accumulator blocks.  Nothing else runs, so the rate is what the matrix units sustain for these
// operand values under the board's power limit.
template <int DT, int MI>
__global__ __launch_bounds__(512) void mfma_probe_kernel(const i32x4* src, float* sink, int iters) {
    typedef abft::Mma<DT, MI> MMA;
    constexpr int TM = 128 / MI, TN = 64 / MI;
    const long long t = (long long)blockIdx.x * 512 + threadIdx.x;
    i32x4 a[TM], b[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) a[i] = src[t * 16 + i];
#pragma unroll
    for (int j = 0; j < TN; ++j) b[j] = src[t * 16 + TM + j];
    typename MMA::Acc acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < MMA::NACC; ++r) acc[i][j][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = MMA::run(a[i], b[j], acc[i][j]);
    }
    typename MMA::AccT total = 0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < MMA::NACC; ++r) total += acc[i][j][r];
    // (no finite sum of these products has this bit pattern's value twice over: never taken)
    if ((float)total == 12345.678f && iters < 0) sink[0] = (float)total;
}

int probe_cus() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return n;
}
}  // namespace

extern "C" {

size_t abft_mfma_probe_bytes(void) {
    const int cus = probe_cus();
    return (size_t)(cus > 0 ? cus : 256) * 512 * 16 * sizeof(i32x4);
}

int abft_mfma_probe(int shape, int dtype, int iters, const void* operands, float* sink, double* ops, void* stream) {
    if (!valid_dtype(dtype) || (shape != 32 && shape != 16)) return ABFT_E_ENUM;
    if (!operands || !sink || !ops) return ABFT_E_NULL;
    if (iters < 1) return ABFT_E_SHAPE;
    const int cus = probe_cus();
    if (cus <= 0) return ABFT_E_HIP;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const i32x4* src = reinterpret_cast<const i32x4*>(operands);
    dim3 grid((unsigned)cus), block(512);
    void (*kern)(const i32x4*, float*, int) = nullptr;
    if (dtype == ABFT_F16) kern = shape == 32 ? mfma_probe_kernel<abft::DT_F16, 32> : mfma_probe_kernel<abft::DT_F16, 16>;
    else if (dtype == ABFT_BF16) kern = shape == 32 ? mfma_probe_kernel<abft::DT_BF16, 32> : mfma_probe_kernel<abft::DT_BF16, 16>;
    else kern = shape == 32 ? mfma_probe_kernel<abft::DT_I8, 32> : mfma_probe_kernel<abft::DT_I8, 16>;
    hipLaunchKernelGGL(kern, grid, block, 0, st, src, sink, iters);
    if (hipGetLastError() != hipSuccess) return ABFT_E_HIP;
    // per wavefront and iteration: 8 MFMAs of 32 x 32 x 16 (16384 multiply-adds each) or 32 of
    // 16 x 16 x 32 (8192 each); int8 shapes are twice as deep
    const double macs = (shape == 32 ? 8.0 * 16384.0 : 32.0 * 8192.0) * (dtype == ABFT_I8 ? 2.0 : 1.0);
    *ops = (double)cus * 8.0 * (double)iters * macs * 2.0;
    return ABFT_OK;
}

void abft_set_kernel_events(void* start_event, void* stop_event) {
    g_ev_start = reinterpret_cast<hipEvent_t>(start_event);
    g_ev_stop = reinterpret_cast<hipEvent_t>(stop_event);
}

}  // extern "C"
