// Which kernel serves which bf16 step.  Steps that have an MFMA kernel use it;
// the rest run the scalar-FMA kernels on bf16 storage.
#include "common.h"
#include <string.h>

namespace beagle {

#ifndef BEAGLE_HAVE_DECODE
size_t decode_bf16_ws_bytes(int32_t M, int32_t, int32_t H, int32_t d, int32_t) {
  return (size_t)2 * M * H * d * sizeof(bf16_t);
}
void launch_decode_bf16(const DecodeArgs& a, hipStream_t s) {
  const int64_t HD = (int64_t)a.H * a.d;
  bf16_t* q = (bf16_t*)a.ws;
  bf16_t* o = q + (int64_t)a.M * HD;
  GemmGroup g; memset(&g, 0, sizeof(g));
  g.count = 1;
  GemmArgs& p = g.p[0];
  p.A = a.x; p.B = a.wq; p.C = q; p.M = a.M; p.N = (int32_t)HD; p.K = a.D;
  p.lda = a.D; p.ldb = HD; p.ldc = HD; p.a_kmajor = 1; p.b_kmajor = 0;
  launch_gemm_bf16_scalar(g, s, "draft_proj_q");
  AttnArgs t; memset(&t, 0, sizeof(t));
  t.B = 1; t.S = a.M; t.L = a.L; t.H = a.H; t.G = a.G; t.d = a.d; t.scale = a.scale;
  t.mask.k = 1; t.mask.eps = 0; t.mask.seq_kv = a.L; t.mask.all_visible = 1;
  t.q = q; t.k = a.kc; t.v = a.vc; t.o = o; t.lse = a.lse;
  launch_attn_fwd_bf16_scalar(t, s);
  p.A = o; p.B = a.wo; p.C = a.y; p.M = a.M; p.N = a.D; p.K = (int32_t)HD;
  p.lda = HD; p.ldb = a.D; p.ldc = a.D;
  launch_gemm_bf16_scalar(g, s, "draft_proj_out");
}
#endif

}  // namespace beagle
