// Run-time specialisation of the persistent recurrent-step kernel (see jit.cpp).
#pragma once
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "kernels.h"
#include "plan.h"
#include "step_layout.h"

namespace rnng {

// HIP source of the step kernel specialised for one component and direction.
std::string jit_step_source(const Plan& P, const CompPlan& cp, bool backward, int NB);
// Same for the wave-autonomous variant with G workgroups; empty if the component is not eligible.
std::string jit_wave_source(const Plan& P, const CompPlan& cp, bool backward, int N, int G);
// Chain of recurrent components side by side in one launch, member g with G[g] <= 32 workgroups
// (members: a chain's members, or its launch with helper members: ChainPlan::fwd_split / bwd_split);
// empty if a member is not eligible for the wave-autonomous variant.
std::string jit_chain_source(const Plan& P, const std::vector<CompPlan>& members, bool backward, int N, const std::vector<int>& G);
// Matrix-core variant for many streams; *lds_bytes receives the dynamic LDS size.
// G unit chunks x J stream groups (N / J streams each).
// *rows receives the accumulator rows per workgroup (tasks x units per chunk).
// *threads: threads per workgroup of the launch (512 where eight wavefronts fit, else 256);
// *blocked: the kernel exchanges through the tile-blocked twins of the shared tensors.
std::string jit_mstep_source(const Plan& P, const CompPlan& cp, bool backward, int N, int G, int J, size_t* lds_bytes, int* rows = nullptr,
                             int* threads = nullptr, bool* blocked = nullptr);
// Matrix-core variant with the two-dimensional split (row groups of GJ workgroups that share
// the columns of every source; partial sums travel through a tensor of *partial_floats floats per frame).
std::string jit_mstep2_source(const Plan& P, const CompPlan& cp, bool backward, int N, int G, int GJ, size_t* lds_bytes,
                              int64_t* partial_floats);
// Chain of matrix-core components in one launch: member g on G[g] unit chunks x J[g] stream groups
// (at most 256 workgroups in all); members: a chain's members, or its backward launch with helper
// members (ChainPlan::bwd_split).  Empty if some member is not eligible.
std::string jit_mstep_chain_source(const Plan& P, const std::vector<CompPlan>& members, bool backward, int N, const std::vector<int>& G,
                                   const std::vector<int>& J, size_t* lds_bytes, int* threads = nullptr, bool* blocked = nullptr);
// Streaming variant (N <= 8 streams; weights read from memory every step, for layers too wide to
// keep on chip): G unit chunks.  *transposed: the kernel reads transposed copies of some matrices.
std::string jit_sstep_source(const Plan& P, const CompPlan& cp, bool backward, int N, int G, size_t* lds_bytes, bool* transposed);
// The same for N >= 9 streams on the matrix cores.
std::string jit_smstep_source(const Plan& P, const CompPlan& cp, bool backward, int N, int G, size_t* lds_bytes, bool* transposed, bool* blocked = nullptr,
                              int* threads = nullptr);
// Compiles (or finds in the process-wide cache) the source; false if hiprtc is missing or the
// compile fails (the log, if any, goes to *log).  Needs no GPU.
bool jit_compile(const std::string& source, std::string* log);
// True if the run-time compiler can be loaded on this machine (else only the interpreting build exists).
bool jit_available();
// Loaded kernel for the source on the current device, or nullptr with the reason (compiler log,
// loader error) in *err.  allow_load = false: only a kernel that is already loaded is returned
// (nothing is compiled or loaded, so no memory is allocated).
// max_dynamic_lds: the most dynamic LDS a launch of the kernel may ask for.
hipFunction_t jit_step_function(const std::string& source, std::string* err, bool allow_load = true, unsigned max_dynamic_lds = STEP_LDS_LIMIT);
hipError_t jit_launch(hipFunction_t fn, StepArgs& a, const StepLaunchPlan& lp, hipStream_t stream);

void fill_step_args(StepArgs& a, const PlanView& pv, const StepLaunchPlan& lp, int desc_off, const float* weights,
                    unsigned* ctrl, int T, int N, bool backward, int spin_limit, int t_begin, int t_end);

}  // namespace rnng
