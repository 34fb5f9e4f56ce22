// Kernel wrappers (generic, one launch per stage) around the device functions of
// accept_dev.h: verification with tolerance, continuation, KV compaction, top-k.
#include "accept_dev.h"

__global__ __launch_bounds__(256) void k_accept(Dims D, DevState s, int tau, int ignore_eos) {
    dev_accept(D, s, blockIdx.x, tau, ignore_eos);
}
void launch_accept(const Dims& D, const DevState& s, int tau, int ignore_eos, hipStream_t st) {
    hipLaunchKernelGGL(k_accept, dim3(D.B), dim3(256), 0, st, D, s, tau, ignore_eos);
}

template <class T>
__global__ __launch_bounds__(256) void k_finalize(Dims D, DevState s, int seq0, int prefill_mode, int ignore_eos) {
    dev_finalize<T>(D, s, seq0 + blockIdx.x, prefill_mode, ignore_eos, 0);
}
void launch_finalize(const Dims& D, const DevState& s, int seq0, int nseq, int prefill_mode, int ignore_eos, int dtype, hipStream_t st) {
    if (dtype) hipLaunchKernelGGL(k_finalize<bf16_t>, dim3(nseq), dim3(256), 0, st, D, s, seq0, prefill_mode, ignore_eos);
    else hipLaunchKernelGGL(k_finalize<float>, dim3(nseq), dim3(256), 0, st, D, s, seq0, prefill_mode, ignore_eos);
}

// grid (nH, nseq, Ly), 64 threads; runs after k_finalize
template <class T>
__global__ __launch_bounds__(64) void k_commit_kv(Dims D, DevState s, int seq0) {
    dev_commit_kv<T>(D, s, blockIdx.z, seq0 + blockIdx.y, blockIdx.x, threadIdx.x);
}
void launch_commit_kv(const Dims& D, const DevState& s, int seq0, int nseq, int dtype, hipStream_t st) {
    dim3 grid(D.nH, nseq, D.Ly), blk(64);
    if (dtype) hipLaunchKernelGGL(k_commit_kv<bf16_t>, grid, blk, 0, st, D, s, seq0);
    else hipLaunchKernelGGL(k_commit_kv<float>, grid, blk, 0, st, D, s, seq0);
}

__global__ __launch_bounds__(256) void k_topk(Dims D, DevState s, int seq0) {
    dev_topk<true>(D, s, blockIdx.x, seq0 + blockIdx.y);
}
void launch_topk(const Dims& D, const DevState& s, int seq0, int nseq, hipStream_t st) {
    hipLaunchKernelGGL(k_topk, dim3(D.Hh, nseq), dim3(256), 0, st, D, s, seq0);
}
