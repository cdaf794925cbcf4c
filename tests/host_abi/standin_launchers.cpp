// Stand-ins for the kernel launchers: they record that a launch was requested and return success, so
// that the C ABI's host code can be exercised without a GPU.  Sizes are the real formulas where the ABI
// compares them with the scratch buffer.
#include "kernels.hpp"

size_t hip_standin_live_allocations = 0;
size_t hip_standin_fail_after = (size_t)-1;
extern "C" { int standin_launches = 0; }

namespace csk {
static hipError_t ok() { ++standin_launches; return hipSuccess; }
hipError_t launch_sketch(const OpDesc&, const float*, int, float*, hipStream_t) { return ok(); }
hipError_t launch_sketch_multi(const OpDesc*, int, const float*, int, float*, hipStream_t, void*, size_t) { return ok(); }
bool sketch_srht_supported(const OpDesc& op) { return op.nbits <= 15; }
hipError_t launch_plan_build(const Plan&, const float*, hipStream_t) { return ok(); }
size_t recover_spill_floats(const Plan& p, int k, int) { return p.N > 512 || k > 64 ? (size_t)k * p.rb * p.N : 0; }
hipError_t launch_recover(const Plan&, const RecoverArgs&, int, hipStream_t) { return ok(); }
bool recover_iht_supported(const Plan& p, int k, int) { return p.rb == 1 && k <= 64 && p.N <= 512; }
hipError_t launch_recover_iht(const Plan&, const RecoverArgs&, int, int, hipStream_t) { return ok(); }
bool recover_inc_supported(const Plan& p, int k, int) { return p.rb == 1 && k <= 64 && p.N <= 512; }
hipError_t launch_recover_inc(const Plan&, const RecoverArgs&, const IncArgs&, int, hipStream_t) { return ok(); }
size_t recover_inc_state_words(int k) { return (size_t)((2 + k + k * k + 3) & ~3); }
hipError_t launch_recover_carry(const Plan&, const RecoverArgs&, const IncArgs&, int, hipStream_t) { return ok(); }
hipError_t launch_backproject(const OpDesc&, const float*, float*, hipStream_t) { return ok(); }
hipError_t launch_topk(const float*, int, int, int32_t*, hipStream_t) { return ok(); }
size_t pool_rows_scratch_floats(int m, int k_tok) { return (size_t)m * ((k_tok + 63) / 64); }
hipError_t launch_pool_rows(const float*, int, int, const int32_t*, int, float*, float*, float*, hipStream_t) { return ok(); }
size_t softmax_entropy_scratch_floats(int B, int V) { return (size_t)B * ((V + 8191) / 8192) * 3; }
hipError_t launch_softmax_entropy(const float*, int, int, float*, float*, hipStream_t) { return ok(); }
hipError_t launch_gather_rows(const void*, int, size_t, const int32_t*, int, void*, hipStream_t) { return ok(); }
hipError_t launch_zero_fill(void*, size_t, hipStream_t) { return ok(); }
hipError_t launch_stream_read(const void*, size_t, uint32_t*, hipStream_t) { return ok(); }
size_t ffn_scratch_bytes(const FfnArgs& a) {
    if (a.T <= 16) return (size_t)a.G * 16 * a.b * 2 + 8208;
    return (size_t)a.T * a.k * a.b * 4;
}
bool ffn_gemm_ok(const FfnArgs&) { return false; }
size_t ffn_gemm_scratch_bytes(const FfnArgs&) { return 0; }
hipError_t launch_ffn_gemm(const FfnArgs&, hipStream_t) { return ok(); }
bool ffn_wide_ok(const FfnArgs&) { return false; }
size_t ffn_wide_scratch_bytes(const FfnArgs&) { return 0; }
hipError_t launch_ffn_wide(const FfnArgs&, hipStream_t) { return ok(); }
hipError_t launch_block_ffn(const FfnArgs&, hipStream_t) { return ok(); }
size_t attn_scratch_bytes(const AttnArgs& a) { return (size_t)a.B * a.kh * 32 * (a.dh + 2) * 4; }
hipError_t launch_head_attn(const AttnArgs&, hipStream_t) { return ok(); }
}  // namespace csk
