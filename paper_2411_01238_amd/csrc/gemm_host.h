// Host-side declarations shared by the GEMM translation units: the launch heuristics and knobs (defined in
// sdrop_gemm.hip) and the two entry functions that each typed translation unit (sdrop_gemm_f16.hip,
// sdrop_gemm_bf16.hip) instantiates for its operand type.  The kernels are compiled per operand type in
// separate files so that they build in parallel.
#ifndef SDROP_GEMM_HOST_H
#define SDROP_GEMM_HOST_H
#include "gemm_device_common.h"

namespace sdrop {

// Kernels with the element-wise tail are separate instantiations, so that eq. (1)-(3) proper run
// exactly the code they would without it.
inline bool has_tail(const GemmParams &P) { return P.bias != nullptr || P.aux != nullptr || P.act != 0 || P.C2 != nullptr; }

// The persistent kernels are compiled once per kind of tail: the common ones each have a form that
// holds that tail's code only (see Compute::store), everything else runs the generic form.
enum TailMode {
    kTailNone = 0,        // eq. (1)-(3) proper
    kTailLight,           // bias and/or ReLU (or neither, with a second output), no gate
    kTailReluGate,        // ReLU gate, no activation (bias allowed)
    kTailGeluErf,         // GELU (erf form), no gate
    kTailGeluErfGate,     // that GELU's derivative as the gate, no activation
    kTailGeneric          // anything else (the tanh form, an activation together with a gate)
};
inline int tail_mode(const GemmParams &P)
{
    if (!has_tail(P)) return kTailNone;
    if (P.aux == nullptr) {
        if (P.act == SDROP_ACT_NONE || P.act == SDROP_ACT_RELU) return kTailLight;
        return P.act == SDROP_ACT_GELU_ERF ? kTailGeluErf : kTailGeneric;
    }
    if (P.act != SDROP_ACT_NONE) return kTailGeneric;
    return P.gate_mode == SDROP_GATE_RELU ? kTailReluGate : P.gate_mode == SDROP_GATE_GELU_ERF ? kTailGeluErfGate : kTailGeneric;
}

// dX: width of the tiles, and whether the persistent kernel computes them (see sdrop_gemm.hip)
struct DxPlan { int TN; bool persistent; bool pairs; };
// fused: the plan is for sdrop_bwd's single launch, whose dW workgroups fill what dX's last round leaves idle
DxPlan dx_plan(const GemmParams &P, bool fused = false);
// [N,K] weights: does the call's kernel read the array in place?
bool w_nk_native(int op, int64_t N, int BM, int BK);
// dW with 64-row tiles: the persistent kernel from 16 expected slices per tile on
bool dw64_persistent(const GemmParams &P);

// which single launch sdrop_bwd uses (see run_bwd)
enum BwdForm { kBwdNone = 0, kBwdPersistent, kBwdTile128, kBwdTile64 };
// the tile width argument of bwd_fused_typed that stands for 256-wide tiles from the pair list
constexpr int kTNPairs = 257;
// ... and the one for single-block tiles with the weight read, and its gradient written, as [N,K]
constexpr int kTNNK = 129;

// One of the three products for operands of type T: picks tile shapes and kernel form, launches.
// o32: fp32 output instead of the operands' type.
template <class T> int dispatch_typed(int op, bool o32, GemmParams &P, hipStream_t stream);
// Both gradients in one launch, in the given form; dw_f32: dW's launch writes fp32 planes (a split reduction).
// Returns -1 when the device does not grant the LDS the launch needs.
template <class T> int bwd_fused_typed(int form, int TN, bool o32, bool dw_f32, const GemmParams &Pdx, const GemmParams &Pdw,
                                       int n_dx, hipStream_t stream);
// The forward product by the kernel that draws its own mask and writes the mask object (see gemm_seeded_grid.h).
// Returns -1 when the device does not grant the LDS the launch needs.
template <class T> int fwd_seeded_typed(bool o32, const GemmParams &P, hipStream_t stream);
extern template int fwd_seeded_typed<F16>(bool, const GemmParams &, hipStream_t);
extern template int fwd_seeded_typed<BF16>(bool, const GemmParams &, hipStream_t);
extern template int dispatch_typed<F16>(int, bool, GemmParams &, hipStream_t);
extern template int dispatch_typed<BF16>(int, bool, GemmParams &, hipStream_t);
extern template int bwd_fused_typed<F16>(int, int, bool, bool, const GemmParams &, const GemmParams &, int, hipStream_t);
extern template int bwd_fused_typed<BF16>(int, int, bool, bool, const GemmParams &, const GemmParams &, int, hipStream_t);

}  // namespace sdrop
#endif
