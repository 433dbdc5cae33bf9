// Tile configurations shared by the host-side dispatcher and the kernel instantiations.
#pragma once
#include "gemm_kernel.h"

namespace abft {

// Index into the configuration table.
//  F* run the direct-to-LDS kernel (16-byte aligned operands and leading dimensions, K a multiple of 128 bytes):
//    F256W  256 x 256, wavefronts 2 x 4 of 128 x  64 (two per SIMD), 2 LDS stages   compute-bound products;
//                                                                    16x16x32 MFMA shapes (the others 32x32x16): no
//                                                                    wavefront-level scheme runs on it
//    F256N  256 x 128, wavefronts 4 x 2 of  64 x  64, 3 stages, 16x16x32 shapes       about one tile per compute unit,
//                                                                    unprotected / global
//    F256S  256 x  64, wavefronts 8 x 1 of  32 x  64, 3 stages, 16x16x32 shapes       outputs of at most 64 columns
//                                                                    (many rows), unprotected / global
//    F128   128 x 128, wavefronts 2 x 2 of  64 x  64, 2 stages       mid-size, unprotected / global
//    F128E  128 x 128, wavefronts 4 x 2 of  32 x  64 (two per SIMD), 3 stages, 16x16x32 shapes
//                                                                    at most one such tile per compute unit: the second
//                                                                    wavefront per SIMD and the third stage stand in for
//                                                                    the second workgroup that would hide the latencies;
//                                                                    unprotected / global
//    F128T  128 x 128, wavefronts 4 x 1 of  32 x 128, 2 stages       thread-level (wide tiles: two checksum
//                                                                    MFMAs per four), narrow outputs, K of one k tile
//    F64T    64 x 128, wavefronts 2 x 1 of  32 x 128, 3 stages       between the streaming tiles and F128
//  S* run the streaming kernel (same alignment, K any multiple of 16 bytes; four wavefronts split the k tiles of one
//  register tile between them, each with its own LDS stages, no barrier in the k loop):
//    S32     32 x  32, 4 stages per wavefront                         a few tiles only: latency-bound layers
//    S64     32 x  64, 3 stages per wavefront
//    S128    64 x  64, 2 stages per wavefront                         up to about one tile per compute unit
//  G* run the generic kernel (any alignment, layout, K):
//    G128 128 x 128, G64 64 x 64 (32x32 MFMA shapes), G16 16 x 64 (16x16 shapes; M <= 16)
enum CfgId { CFG_F256W = 0, CFG_F128, CFG_F128T, CFG_F64T, CFG_S32, CFG_S64, CFG_S128, CFG_G128, CFG_G64, CFG_G16, CFG_F256N, CFG_F256S, CFG_F128E, CFG_COUNT };

template <int DT, int ID>
struct CfgOf;
//                                             MI TM TN WM WN BKB
template <int DT> struct CfgOf<DT, CFG_F128>  { typedef Cfg<DT, 32, 2, 2, 2, 2, 128> type; static constexpr int NSTAGE = 2; static constexpr int KWAYS = 1; };
template <int DT> struct CfgOf<DT, CFG_F128T> { typedef Cfg<DT, 32, 1, 4, 4, 1, 128> type; static constexpr int NSTAGE = 2; static constexpr int KWAYS = 1; };
template <int DT> struct CfgOf<DT, CFG_F64T>  { typedef Cfg<DT, 32, 1, 4, 2, 1, 128> type; static constexpr int NSTAGE = 3; static constexpr int KWAYS = 1; };
template <int DT> struct CfgOf<DT, CFG_F256W> { typedef Cfg<DT, 16, 8, 4, 2, 4, 128> type; static constexpr int NSTAGE = 2; static constexpr int KWAYS = 1; };
template <int DT> struct CfgOf<DT, CFG_F256N> { typedef Cfg<DT, 16, 4, 4, 4, 2, 128> type; static constexpr int NSTAGE = 3; static constexpr int KWAYS = 1; };
template <int DT> struct CfgOf<DT, CFG_F256S> { typedef Cfg<DT, 16, 2, 4, 8, 1, 128> type; static constexpr int NSTAGE = 3; static constexpr int KWAYS = 1; };
template <int DT> struct CfgOf<DT, CFG_F128E> { typedef Cfg<DT, 16, 2, 4, 4, 2, 128> type; static constexpr int NSTAGE = 3; static constexpr int KWAYS = 1; };
template <int DT> struct CfgOf<DT, CFG_S32>   { typedef Cfg<DT, 32, 1, 1, 1, 1, 128> type; static constexpr int NSTAGE = 4; static constexpr int KWAYS = 4; };
template <int DT> struct CfgOf<DT, CFG_S64>   { typedef Cfg<DT, 32, 1, 2, 1, 1, 128> type; static constexpr int NSTAGE = 3; static constexpr int KWAYS = 4; };
template <int DT> struct CfgOf<DT, CFG_S128>  { typedef Cfg<DT, 32, 2, 2, 1, 1, 128> type; static constexpr int NSTAGE = 2; static constexpr int KWAYS = 4; };
template <int DT> struct CfgOf<DT, CFG_G128>  { typedef Cfg<DT, 32, 2, 2, 2, 2, 128> type; static constexpr int NSTAGE = 0; static constexpr int KWAYS = 1; };
template <int DT> struct CfgOf<DT, CFG_G64>   { typedef Cfg<DT, 32, 1, 1, 2, 2, 128> type; static constexpr int NSTAGE = 0; static constexpr int KWAYS = 1; };
template <int DT> struct CfgOf<DT, CFG_G16>   { typedef Cfg<DT, 16, 1, 1, 1, 4, 256> type; static constexpr int NSTAGE = 0; static constexpr int KWAYS = 1; };

constexpr bool cfg_is_stream(int id) { return id == CFG_S32 || id == CFG_S64 || id == CFG_S128; }

// threads: of one WAVES_M x WAVES_N grid of wavefronts (a streaming launch has kways times as many);
// kway_bytes: bytes of k that one wavefront takes in turn when kways wavefronts share a tile
struct CfgInfo {
    int bm, bn, bk_bytes, wm, wn, threads, lds_bytes, fast, kways, kway_bytes, mi;
};

template <int ID>
constexpr CfgInfo cfg_info() {
    typedef typename CfgOf<DT_F16, ID>::type C;  // identical for every dtype (rows / columns / k bytes)
    constexpr int ns = CfgOf<DT_F16, ID>::NSTAGE;
    constexpr int kw = CfgOf<DT_F16, ID>::KWAYS;
    constexpr int lds = cfg_is_stream(ID) ? kw * ns * ((C::BM + C::BN) * 128 + 768)
                                          : (ns ? ns * ((C::BM + C::BN) * 128 + 1024) + 512 : C::LDS_BYTES);
    return CfgInfo{C::BM, C::BN, C::BKB, C::WM, C::WN, C::THREADS, lds, ns ? 1 : 0, kw, cfg_is_stream(ID) ? 128 : 32, C::MI};
}

inline CfgInfo cfg_info_host(int id) {
    switch (id) {
        case CFG_F128: return cfg_info<CFG_F128>();
        case CFG_F128T: return cfg_info<CFG_F128T>();
        case CFG_F64T: return cfg_info<CFG_F64T>();
        case CFG_F256W: return cfg_info<CFG_F256W>();
        case CFG_F256N: return cfg_info<CFG_F256N>();
        case CFG_F256S: return cfg_info<CFG_F256S>();
        case CFG_F128E: return cfg_info<CFG_F128E>();
        case CFG_S32: return cfg_info<CFG_S32>();
        case CFG_S64: return cfg_info<CFG_S64>();
        case CFG_S128: return cfg_info<CFG_S128>();
        case CFG_G128: return cfg_info<CFG_G128>();
        case CFG_G64: return cfg_info<CFG_G64>();
        default: return cfg_info<CFG_G16>();
    }
}

// implemented once per dtype in gemm_f16.hip / gemm_bf16.hip / gemm_i8.hip
hipError_t launch_gemm_f16(int cfg, int mode, bool inject, const GemmArgs& args, hipStream_t stream);
hipError_t launch_gemm_bf16(int cfg, int mode, bool inject, const GemmArgs& args, hipStream_t stream);
hipError_t launch_gemm_i8(int cfg, int mode, bool inject, const GemmArgs& args, hipStream_t stream);

}  // namespace abft
