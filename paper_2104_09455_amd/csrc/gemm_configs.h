// Tile configurations shared by the host-side dispatcher and the kernel instantiations.
#pragma once
#include "gemm_kernel.h"

namespace abft {

// Index into the configuration table.  L/M/S use 32x32 MFMA shapes on square wave
// grids; T is the skinny path (M <= 16: batch-1 inference) on 16x16 shapes.
enum CfgId { CFG_L = 0, CFG_M = 1, CFG_S = 2, CFG_T = 3, CFG_COUNT = 4 };

template <int DT, int ID>
struct CfgOf;
//                                         MI TM TN WM WN BKB
template <int DT> struct CfgOf<DT, CFG_L> { typedef Cfg<DT, 32, 4, 4, 2, 2, 128> type; };
template <int DT> struct CfgOf<DT, CFG_M> { typedef Cfg<DT, 32, 2, 2, 2, 2, 128> type; };
template <int DT> struct CfgOf<DT, CFG_S> { typedef Cfg<DT, 32, 1, 1, 2, 2, 128> type; };
template <int DT> struct CfgOf<DT, CFG_T> { typedef Cfg<DT, 16, 1, 1, 1, 4, 256> type; };

struct CfgInfo {
    int bm, bn, bk_bytes, wm, wn, threads, lds_bytes;
};

template <int DT, int ID>
constexpr CfgInfo cfg_info() {
    typedef typename CfgOf<DT, ID>::type C;
    return CfgInfo{C::BM, C::BN, C::BKB, C::WM, C::WN, C::THREADS, C::LDS_BYTES};
}

// identical for every dtype (tiles are defined in rows / columns / k-bytes)
inline CfgInfo cfg_info_host(int id) {
    switch (id) {
        case CFG_L: return cfg_info<DT_F16, CFG_L>();
        case CFG_M: return cfg_info<DT_F16, CFG_M>();
        case CFG_S: return cfg_info<DT_F16, CFG_S>();
        default: return cfg_info<DT_F16, CFG_T>();
    }
}

// implemented once per dtype in gemm_f16.hip / gemm_bf16.hip / gemm_i8.hip
hipError_t launch_gemm_f16(int cfg, int mode, bool inject, const GemmArgs& args, hipStream_t stream);
hipError_t launch_gemm_bf16(int cfg, int mode, bool inject, const GemmArgs& args, hipStream_t stream);
hipError_t launch_gemm_i8(int cfg, int mode, bool inject, const GemmArgs& args, hipStream_t stream);

}  // namespace abft
