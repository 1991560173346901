// Entry points that launch nothing: version, error names, workspace sizes.
#include "common.hpp"

namespace fastar {
size_t compress_ws_bytes(int H, int C, int n_new, int r);
size_t select_self_ws_bytes(int H, int n_q, int C, int r, int BQ, int BK, int n_rep);
size_t select_cross_ws_bytes(int H, int n_q, int n_p, int BQ);
}  // namespace fastar

extern "C" const char *fastar_version(void) { return "fastar-gfx950 0.1"; }

extern "C" const char *fastar_strerror(int code) {
    switch (code) {
        case FASTAR_OK: return "ok";
        case FASTAR_ERR_INVALID_ARG: return "invalid argument";
        case FASTAR_ERR_UNSUPPORTED: return "unsupported shape or type";
        case FASTAR_ERR_WORKSPACE: return "workspace too small";
        case FASTAR_ERR_HIP: return "HIP launch error";
        default: return "unknown error";
    }
}

extern "C" size_t fastar_workspace_bytes(int op, int H, int n_q, int n_k, int r, int BQ, int BK, int n_rep) {
    switch (op) {
        case FASTAR_OP_COMPRESS: return fastar::compress_ws_bytes(H, n_k, n_q, r);
        case FASTAR_OP_SELECT_SELF: return fastar::select_self_ws_bytes(H, n_q, n_k, r, BQ, BK, n_rep);
        case FASTAR_OP_SELECT_CROSS: return fastar::select_cross_ws_bytes(H, n_q, n_k, BQ);
        default: return 0;
    }
}
