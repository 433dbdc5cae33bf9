// A chain of fully-connected layers in ONE launch (Sec. 2.4 step 4: layer l's output, after its
// activation function, is layer l + 1's input), for the latency-bound MLPs of recommendation
// models: every layer protected by its own scheme, the activations never leave the L2.
//
// MI355X has eight dies (XCDs), each with 32 compute units and an L2 of its own; anything that
// crosses dies goes through memory and costs microseconds, the time of a whole layer here.  So the
// batch is cut into eight slabs of rows, one per die: a die runs ALL layers for its rows, streaming
// the weights itself (they come out of the memory-side cache), and the layers of a slab are chained
// through that die's L2 alone.  Workgroups are dealt to the dies round-robin (from a starting die
// that varies between queues, so a workgroup asks the hardware which die it is on; the eight
// workgroups b with the same b / 8 land on eight different dies, which makes b / 8 its rank among
// the 32 of its die), the 32 workgroups of a die share out the 32 x 32 output tiles of each layer,
// and a layer's tiles wait for the previous layer of the same slab through completion flags: plain
// stores, and loads that go past the compute unit's cache to the die's L2; no atomics (those are
// executed at the memory side).  A flag flips once per launch (sense reversal), so nothing has to
// be cleared between launches.
//
// Each tile is computed by the streaming kernel's tile routine: same arithmetic, same checks, same
// fault flag as a launch per layer.
#pragma once
#include "gemm_configs.h"
#include "gemm_stream.h"

namespace abft {

constexpr int CHAIN_MAX_LAYERS = 8;
constexpr int CHAIN_DIES = 8;
constexpr int CHAIN_TEAM = 32;                       // workgroups per die
constexpr int CHAIN_FLAG_WORDS = CHAIN_DIES * CHAIN_MAX_LAYERS * CHAIN_TEAM;
// status bits (device word owned by the plan)
constexpr unsigned CHAIN_TIMEOUT = 1u;               // a wait for the previous layer ran out of spins
constexpr unsigned CHAIN_WRONG_DIE = 2u;             // the hardware reported a die id outside 0..7

struct ChainLayer {
    const char* A;            // input: the caller's for the first layer, else the previous layer's C
    const char* B;            // weights, N x K (k contiguous)
    char* C;
    int N, K;
    long long lda, ldb, ldc;  // elements
    const char* beta_k;       // global scheme: weight checksums per block of 32 columns (see GemmArgs)
    const char* beta_p;
    int mode;                 // MODE_NONE, MODE_GLOBAL or MODE_THREAD
    int act;                  // activation function applied to the stored values
    int depends;              // A is the previous layer's C: wait for it
    double tol_coeff, tol_l1;
};

struct ChainArgs {
    ChainLayer layer[CHAIN_MAX_LAYERS];
    int n_layers, M;
    unsigned* flags;          // [die][layer][workgroup of the die]: flips when that workgroup is done with the layer
    unsigned* status;         // CHAIN_* bits, sticky
    unsigned* fault_flag;
    int spin_limit;           // polls of one wait before it gives up
};

// loads that go past the compute unit's cache (device scope: served by the die's L2)
__device__ __forceinline__ unsigned load_past_l1(const unsigned* p) {
    unsigned v;
    asm volatile("global_load_dword %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
    return v;
}
// id of the die (XCC) this wavefront runs on: hardware register XCC_ID, bits 3:0
__device__ __forceinline__ unsigned die_id() { return __builtin_amdgcn_s_getreg((31 << 11) | 20) & 15u; }

template <int DT>
__global__ __launch_bounds__(256) void mlp_chain_kernel(const ChainArgs a) {
    typedef typename CfgOf<DT, CFG_S32>::type CFG;   // 32 x 32 tiles, four wavefronts sharing the k loop
    constexpr int NST = CfgOf<DT, CFG_S32>::NSTAGE;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ int s_abort;
    __shared__ unsigned s_target;

    const int tid = threadIdx.x;
    const unsigned die = die_id();
    const int rank = (int)blockIdx.x / CHAIN_DIES;   // of this workgroup among those of its die
    if (die >= (unsigned)CHAIN_DIES) {
        if (tid == 0) {
            atomicOr(a.status, CHAIN_WRONG_DIE);
            atomicOr(a.fault_flag, 1u);
        }
        return;
    }
    // the rows of this die: whole tile rows, the same number for every die
    const int tiles_m_all = (a.M + 31) / 32;
    const int slab_tiles = (tiles_m_all + CHAIN_DIES - 1) / CHAIN_DIES;
    const int tm0 = (int)die * slab_tiles;
    const int tm1 = tm0 + slab_tiles < tiles_m_all ? tm0 + slab_tiles : tiles_m_all;
    if (tm0 >= tm1) return;                          // no rows left for this die (all of its workgroups leave)
    unsigned* const fl = a.flags + (size_t)die * CHAIN_MAX_LAYERS * CHAIN_TEAM;
    if (tid == 0) s_abort = 0;
    __syncthreads();

    // wavefront 0 waits until all 32 workgroups of the die have flipped their flag of layer `l` to
    // `target` (lane r polls workgroup r's flag); a bounded number of polls, then the launch gives up
    auto wait_for_layer = [&](int l, unsigned target) {
        if (tid >= 64) return;
        int spins = 0;
        for (;;) {
            const unsigned f = tid < CHAIN_TEAM ? load_past_l1(fl + l * CHAIN_TEAM + tid) : target;
            if (__all(f == target)) break;
            if (++spins > a.spin_limit) {
                if (tid == 0) {
                    atomicOr(a.status, CHAIN_TIMEOUT);
                    atomicOr(a.fault_flag, 1u);   // what this launch leaves behind is not to be trusted
                    s_abort = 1;
                }
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
    };

    unsigned prev_target = 0;
    for (int l = 0; l < a.n_layers; ++l) {
        const ChainLayer& L = a.layer[l];
        // this launch's value of the layer's flags: the opposite of what this workgroup left there
        if (tid == 0) s_target = load_past_l1(fl + l * CHAIN_TEAM + rank) ^ 1u;
        if (L.depends && l > 0) wait_for_layer(l - 1, prev_target);
        __syncthreads();
        if (s_abort) return;                         // (uniform: every wavefront of the workgroup leaves)
        const unsigned target = s_target;

        GemmArgs g;
        g.A = L.A; g.B = L.B; g.C = L.C;
        g.M = a.M; g.N = L.N; g.K = L.K;
        g.lda = L.lda; g.ldb = L.ldb; g.ldc = L.ldc;
        g.b_sn = L.ldb; g.b_sk = 1;
        g.a_vec = g.b_vec = 1;
        g.conv = 0;
        g.beta_k = L.beta_k; g.beta_p = L.beta_p; g.beta_r = nullptr;
        g.partial_dots = nullptr; g.n_parts = 0;
        g.tol_l1 = L.tol_l1; g.tol_coeff = L.tol_coeff;
        g.flag = a.fault_flag; g.report = nullptr;
        g.f_row = g.f_col = -1; g.f_bit = 0; g.f_kt = -1;
        g.tiles_m = tiles_m_all; g.tiles_n = (L.N + 31) / 32;
        g.act = L.act;
        g.alpha_out = nullptr; g.ld_alpha_out = 0; g.alpha_in = nullptr;
        const int ntiles = (tm1 - tm0) * g.tiles_n;
        for (int t = rank; t < ntiles; t += CHAIN_TEAM) {
            const int tile_m = tm0 + t / g.tiles_n, tile_n = t % g.tiles_n;
            __syncthreads();                         // the previous tile is done with the LDS
            // (inputs written by other compute units in this launch: read past this one's cache)
            if (L.mode == MODE_GLOBAL) stream_tile<CFG, NST, MODE_GLOBAL, false, false, false, true>(g, tile_m, tile_n, smem);
            else if (L.mode == MODE_THREAD) stream_tile<CFG, NST, MODE_THREAD, false, false, false, true>(g, tile_m, tile_n, smem);
            else stream_tile<CFG, NST, MODE_NONE, false, false, false, true>(g, tile_m, tile_n, smem);
        }
        // this workgroup's stores of C have reached the L2; then its flag of the layer flips
        __builtin_amdgcn_s_waitcnt(0);               // vmcnt(0), expcnt(0), lgkmcnt(0)
        __syncthreads();
        if (tid == 0) *reinterpret_cast<volatile unsigned*>(fl + l * CHAIN_TEAM + rank) = target;
        prev_target = target;
    }
    // Every rank of the die must have been there: were the workgroups not dealt out as assumed, a
    // rank would be missing on some die, its tiles undone and its flag unflipped -- seen here (and in
    // the waits above) as a time-out, never silently.
    wait_for_layer(a.n_layers - 1, prev_target);
}

hipError_t launch_mlp_chain_f16(const ChainArgs& args, hipStream_t stream);
hipError_t launch_mlp_chain_bf16(const ChainArgs& args, hipStream_t stream);

}  // namespace abft
