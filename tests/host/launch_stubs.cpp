// Stand-ins for the kernel launchers so that the C ABI's host logic can be linked and run without device code.
#include "hy_launch.hpp"

namespace hy {
hy_status launch_stencil(const ConvPtrs*, int, const ConvShape& s, hipStream_t) { return s.lh > 8 ? HY_ERR_UNSUPPORTED : HY_OK; }
hy_status launch_direct(const ConvPtrs*, int, const ConvShape&, hipStream_t) { return HY_OK; }
hy_status launch_mr_mfma(const ConvPtrs&, const ConvShape& s, hipStream_t) {
    return (s.dtype == HY_BF16 && s.group % 16 == 0 && s.D % 64 == 0 && s.lh <= 513) ? HY_OK : HY_ERR_UNSUPPORTED;
}
bool se_walk_preferred(const ConvShape&, int) { return false; }
hy_status launch_se_walk(const ConvPtrs*, int, const ConvShape&, hipStream_t) { return HY_OK; }
bool cp4_supported(const ConvShape& s) { return s.dtype == HY_BF16 && s.gated && s.D % 128 == 0 && s.lh <= 129; }
hy_status launch_cp4(const ConvPtrs&, const ConvShape& s, hipStream_t) { return cp4_supported(s) ? HY_OK : HY_ERR_UNSUPPORTED; }
bool cp_mfma_supported(const ConvShape& s) { return s.dtype == HY_BF16 && s.gated && s.D % 64 == 0 && s.lh <= 145; }
hy_status launch_cp_mfma(const ConvPtrs&, const ConvShape& s, hipStream_t) { return cp_mfma_supported(s) ? HY_OK : HY_ERR_UNSUPPORTED; }
bool li_mfma_supported(const LiShape& s) { return s.dtype == HY_BF16 && s.group % 16 == 0 && s.D % 64 == 0 && s.order <= 16; }
int64_t li_workspace_bytes(const LiShape& s) { return li_mfma_supported(s) ? s.B * ((s.L + 511) / 512 - 1) * (s.D / 16) * 1024 : 0; }
hy_status launch_li_mfma(const LiPtrs&, const LiShape&, void*, hipStream_t) { return HY_OK; }
hy_status launch_li_direct(const LiPtrs&, const LiShape& s, hipStream_t) { return s.order <= 64 ? HY_OK : HY_ERR_UNSUPPORTED; }
int64_t li_state_workspace_bytes(const LiShape& s) { return li_mfma_supported(s) ? s.B * ((s.L + 511) / 512) * (s.D / 16) * 1024 : 0; }
hy_status launch_li_state(const LiPtrs&, const LiShape&, void*, hipStream_t) { return HY_OK; }
hy_status launch_li_state_fold(const float*, int64_t, int64_t, const float*, const float*, float*, int64_t, int64_t, int32_t, int32_t, hipStream_t) { return HY_OK; }
bool chain4_supported(const ChainShape& s) {
    return s.dtype == HY_BF16 && s.group % 16 == 0 && s.D % 128 == 0 && s.lh <= 129 && s.lf >= 1 && s.lf <= 9;
}
hy_status launch_chain4(const ChainPtrs&, const ChainShape&, hipStream_t) { return HY_OK; }
bool bwd_stencil_supported(const BwdShape& s) { return s.lh <= 8 && s.D % (s.dtype == HY_BF16 ? 2 : 1) == 0; }
int64_t bwd_stencil_workspace_bytes(const BwdShape& s) { return s.B * ((s.L + 127) / 128) * s.D * s.lh * 4; }
hy_status launch_bwd_stencil(const BwdPtrs&, const BwdShape&, void*, hipStream_t) { return HY_OK; }
bool bwd_walk_preferred(const BwdShape&) { return false; }
int64_t bwd_walk_workspace_bytes(const BwdShape& s) { return s.B * s.D * s.lh * 4; }
hy_status launch_bwd_walk(const BwdPtrs&, const BwdShape&, void*, hipStream_t) { return HY_OK; }
hy_status launch_bwd_direct(const BwdPtrs&, const BwdShape&, hipStream_t) { return HY_OK; }
bool mr_bwd_supported(const BwdShape& s) { return s.dtype == HY_BF16 && s.group % 16 == 0 && s.D % 64 == 0 && s.lh > 8 && s.lh <= 129; }
int64_t mr_bwd_rows(const BwdShape& s) { return (s.L + 31) / 32 * 32; }
int64_t mr_bwd_workspace_bytes(const BwdShape& s) { return s.B * (s.D / 16) * s.lh * 4; }
hy_status launch_mr_bwd(const BwdPtrs&, const BwdShape&, void*, hipStream_t) { return HY_OK; }
bool cp4_bwd_supported(const BwdShape& s) { return s.dtype == HY_BF16 && s.D % 128 == 0 && s.lh > 8 && s.lh <= 129; }
int64_t cp4_bwd_workspace_bytes(const BwdShape& s) { return s.B * s.D * s.lh * 4; }
hy_status launch_cp4_bwd(const BwdPtrs&, const BwdShape&, void*, hipStream_t) { return HY_OK; }
hy_status launch_dh_reduce(const float*, float*, int64_t, int64_t, int32_t, int32_t, hipStream_t) { return HY_OK; }
hy_status launch_stream_gate(const void*, const void*, const void*, void*, int64_t, int64_t, int64_t, int32_t, int64_t,
                             int32_t, int32_t, hipStream_t) { return HY_OK; }
hy_status launch_bwd_zero_dh(float*, int64_t, int32_t, int32_t, hipStream_t) { return HY_OK; }
}  // namespace hy
