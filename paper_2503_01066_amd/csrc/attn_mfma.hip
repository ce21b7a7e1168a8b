// Matrix-core attention kernels (placeholder dispatch until the MFMA kernels land).
#include "kernels.h"

namespace alch {

bool attn_mfma_supported(const AttnArgs&) { return false; }
int launch_attn_bwd_mfma(const AttnArgs&, hipStream_t) { return fail(ALCH_ERR_UNSUPPORTED, "no matrix-core attention kernel for this shape"); }

int launch_attn_fwd(alch_dtype dt, const void* Q, const void* K, const void* V, void* O, float* LSE, int T,
                    int n_seqs, int max_seqlen, const int* cu_seqlens, const int* cu_seqlens_host, int Hq,
                    int Hkv, int D, hipStream_t stream) {
    (void)max_seqlen; (void)cu_seqlens_host;
    return launch_attn_fwd_generic(dt, Q, K, V, O, LSE, T, n_seqs, cu_seqlens, Hq, Hkv, D, stream);
}

}  // namespace alch
